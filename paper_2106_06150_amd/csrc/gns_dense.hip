// The update step of one layer (paper Algorithm 1, h_u = g(W . (h_u, h_N(u))), GraphSAGE form of
// Section 2.1), forward only:  out = g([h_self | h_neigh] . W + bias).  This is the one dense
// contraction of the path, so it runs on the matrix cores: fp32 MFMA 32x32x2, fp32 accumulate.
//
// Tiling: a block of 256 threads (4 waves, 2 x 2) owns a 128 x 128 tile of the output and walks K in
// steps of 32.  The A (activations, concatenated on the fly from the two inputs) and B (weights)
// tiles of a step are staged in LDS k-major, so a wave's MFMA operands are 32 consecutive floats of
// one LDS row: lane l feeds A[m = l % 32][k = l / 32] and B[k = l / 32][n = l % 32].  The tiles of the
// next step are fetched into registers while the current step multiplies.  Each wave keeps
// 2 x 2 accumulator tiles of 32 x 32 (64 VGPRs); element v of lane l is row 8*(v/4) + 4*(l/32) + v%4,
// column l % 32 of its tile.
#include "gns_internal.h"
#include "gns_device.hpp"

namespace gns {

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int kDM = 128, kDN = 128, kDK = 32;
constexpr int kDPad = 4;                      // keeps 16-byte alignment of LDS rows, spreads the transposed writes

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

__global__ void __launch_bounds__(kBlock) k_sage_dense(DenseArgs a)
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

    float4 ra[4], rb[4];
    auto fetch = [&](int32_t k0) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int idx = tid + j * kBlock;
            {   // A: 128 rows x 8 float4
                const int row = idx >> 3, k = k0 + (idx & 7) * 4;
                const int64_t gr = (int64_t) m0 + row;
                float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
                if (gr < rows && k < K) {
                    const float* p = (k < a.f1) ? a.a1 + gr * a.f1 + k : a.a2 + gr * a.f2 + (k - a.f1);
                    v = *reinterpret_cast<const float4*>(p);
                }
                ra[j] = v;
            }
            {   // B: 32 k-rows x 32 float4
                const int kr = idx >> 5, n = n0 + (idx & 31) * 4, k = k0 + kr;
                float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
                if (k < K && n < a.hdim) v = *reinterpret_cast<const float4*>(a.w + (int64_t) k * a.hdim + n);
                rb[j] = v;
            }
        }
    };
    auto stage = [&]() {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int idx = tid + j * kBlock;
            const int row = idx >> 3, kc = (idx & 7) * 4;
            As[kc + 0][row] = ra[j].x;
            As[kc + 1][row] = ra[j].y;
            As[kc + 2][row] = ra[j].z;
            As[kc + 3][row] = ra[j].w;
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
    stage();
    __syncthreads();
    const int kh = lane >> 5, l32 = lane & 31;
    for (int32_t k0 = 0; k0 < K; k0 += kDK) {
        const bool more = k0 + kDK < K;
        if (more) fetch(k0 + kDK);
#pragma unroll
        for (int kk = 0; kk < kDK; kk += 2) {
            float af[2], bf[2];
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                af[t] = As[kk + kh][wm * 64 + t * 32 + l32];
                bf[t] = Bs[kk + kh][wn * 64 + t * 32 + l32];
            }
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                for (int nt = 0; nt < 2; ++nt)
                    acc[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[mt], bf[nt], acc[mt][nt], 0, 0, 0);
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
