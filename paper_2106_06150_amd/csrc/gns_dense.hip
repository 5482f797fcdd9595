// The update step of one layer (paper Algorithm 1, h_u = g(W . (h_u, h_N(u))), GraphSAGE form of
// Section 2.1), forward only:  out = g([h_self | h_neigh] . W + bias).  This is the one dense
// contraction of the path, so it runs on the matrix cores: fp32 MFMA 32x32x2, fp32 accumulate.
//
// Tiling: a block of 256 threads (4 waves, 2 x 2) owns a 128 x 128 tile of the output and walks K in
// steps of 32.  The A (activations, concatenated on the fly from the two inputs) and B (weights)
// tiles of a step are staged in LDS; lane l feeds A[m = l % 32][k = l / 32] and
// B[k = l / 32][n = l % 32] of a 32 x 32 product.  A is kept row-major with a row stride of 33 floats,
// B k-major: both the staging writes (a thread's four consecutive k of one row, or its float4 of one
// k-row) and the operand reads (32 consecutive rows of one k, or 32 consecutive columns) then spread
// over the LDS banks.  The tiles of the next step are fetched into registers while the current step
// multiplies, and the operands of step kk + 2 are read before the products of step kk are issued.  Each
// wave keeps 2 x 2 accumulator tiles of 32 x 32 (64 registers); element v of lane l is row
// 8*(v/4) + 4*(l/32) + v%4, column l % 32 of its tile.
#include "gns_internal.h"
#include "gns_device.hpp"

namespace gns {

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int kDM = 128, kDN = 128, kDK = 32;
constexpr int kDFetch = kDM * kDK / 4 / kBlock;  // float4 per thread and operand tile
constexpr int kDPad = 4;                      // B rows: keeps their 16-byte alignment
constexpr int kDAStride = kDK + 1;            // A rows: an odd stride spreads rows over the banks

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
    __shared__ float As[kDM][kDAStride];
    __shared__ float Bs[kDK][kDN + kDPad];
    const int32_t m0 = (int32_t) blockIdx.x * kDM, n0 = (int32_t) blockIdx.y * kDN;
    if (m0 >= a.rows) return;
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
                if (gr < a.rows && k < K) {              // a.rows: what the buffers hold (the device count may be smaller)
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
            const int row = idx / kA4, kc = (idx % kA4) * 4;
            As[row][kc + 0] = ra[j].x;
            As[row][kc + 1] = ra[j].y;
            As[row][kc + 2] = ra[j].z;
            As[row][kc + 3] = ra[j].w;
            const int kr = idx >> 5, nc = (idx & 31) * 4;
            *reinterpret_cast<float4*>(&Bs[kr][nc]) = rb[j];
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
    // the row count read on the device is needed for the early exit and the stores only, so the first
    // fetch does not wait for it
    const int32_t rows = a.rows_dev ? *a.rows_dev : a.rows;
    if (m0 >= rows) return;
    stage();
    __syncthreads();
    const int kh = lane >> 5, l32 = lane & 31;
    for (int32_t k0 = 0; k0 < K; k0 += kDK) {
        const bool more = k0 + kDK < K;
        if (more) fetch(k0 + kDK);
        const float* arow = &As[wm * 64 + l32][kh];
        const float* brow = &Bs[kh][wn * 64 + l32];
        float af[2][2], bf[2][2];
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            af[0][t] = arow[t * 32 * kDAStride];
            bf[0][t] = brow[t * 32];
        }
#pragma unroll
        for (int kk = 0; kk < kDK; kk += 2) {
            const int cur = (kk >> 1) & 1;
            if (kk + 2 < kDK) {
#pragma unroll
                for (int t = 0; t < 2; ++t) {
                    af[cur ^ 1][t] = arow[t * 32 * kDAStride + kk + 2];
                    bf[cur ^ 1][t] = brow[(kk + 2) * (kDN + kDPad) + t * 32];
                }
            }
            __builtin_amdgcn_sched_barrier(0);          // the reads above stay ahead of the products below
            acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[cur][0], bf[cur][0], acc[0][0], 0, 0, 0);
            acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[cur][0], bf[cur][1], acc[0][1], 0, 0, 0);
            acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[cur][1], bf[cur][0], acc[1][0], 0, 0, 0);
            acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[cur][1], bf[cur][1], acc[1][1], 0, 0, 0);
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
