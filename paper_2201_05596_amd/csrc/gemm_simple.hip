// Plain LDS-tiled grouped GEMM with fp32 accumulation on the vector ALUs.
// It serves the fp32 layer (the tiny functional configuration, where launch
// latency is the bound) and bf16 shapes the MFMA kernels do not cover.
//   out[g, r, n] = epi( sum_k A[row(g,r), k] B[g, k, n] + bias[g, n] ),  r < rows(g)
// (paper Sec. 3.1: each expert is an FFN; this is one of its two products.)
#include "moe_internal.h"

namespace moe {

constexpr int kSTile = 64;   // output tile edge
constexpr int kSK = 16;      // k-chunk

template <typename T>
__global__ __launch_bounds__(256) void gemm_simple_kernel(GemmArgs a) {
    __shared__ float As[kSK][kSTile + 1];   // [k][m]
    __shared__ float Bs[kSK][kSTile + 4];   // [k][n]
    __shared__ long long arow[kSTile];      // A-row index per tile row, -1 = inactive

    const int g = blockIdx.z;
    const int rows = a.rows ? min(a.rows[g], a.max_rows) : a.fixed_rows;
    const int m0 = blockIdx.y * kSTile;
    if (m0 >= rows) return;
    const int n0 = blockIdx.x * kSTile;
    const int tid = threadIdx.x;
    const T* A = static_cast<const T*>(a.A);
    const T* B = static_cast<const T*>(a.B) + (size_t)g * a.K * a.N;

    if (tid < kSTile) {
        const int r = m0 + tid;
        long long ar = -1;
        if (r < rows) {
            if (a.row_map) ar = a.row_map[(size_t)g * a.max_rows + r];
            else ar = (long long)g * a.a_group_stride + r;
        }
        arow[tid] = ar;
    }
    __syncthreads();

    const int tm = (tid / 16) * 4, tn = (tid % 16) * 4;
    float acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;

    for (int k0 = 0; k0 < a.K; k0 += kSK) {
        for (int i = tid; i < kSTile * kSK; i += 256) {
            const int m = i / kSK, k = i % kSK;              // A: consecutive threads walk k (contiguous)
            const long long ar = arow[m];
            As[k][m] = (ar >= 0 && k0 + k < a.K) ? Elem<T>::load(A + (size_t)ar * a.K + k0 + k) : 0.f;
        }
        for (int i = tid; i < kSTile * kSK; i += 256) {
            const int k = i / kSTile, n = i % kSTile;        // B: consecutive threads walk n (contiguous)
            Bs[k][n] = (k0 + k < a.K && n0 + n < a.N) ? Elem<T>::load(B + (size_t)(k0 + k) * a.N + n0 + n) : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int k = 0; k < kSK; ++k) {
            float av[4], bv[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) av[i] = As[k][tm + i];
#pragma unroll
            for (int j = 0; j < 4; ++j) bv[j] = Bs[k][tn + j];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(av[i], bv[j], acc[i][j]);
        }
        __syncthreads();
    }

    const T* bias = a.bias ? static_cast<const T*>(a.bias) + (size_t)g * a.N : nullptr;
    T* out = static_cast<T*>(a.out);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int r = m0 + tm + i;
        if (r >= rows || arow[tm + i] < 0) continue;
        T* orow = out + ((size_t)g * a.o_group_stride + r) * a.N;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int n = n0 + tn + j;
            if (n >= a.N) continue;
            float v = acc[i][j] + (bias ? Elem<T>::load(bias + n) : 0.f);
            if (a.gelu) v = gelu_tanh(v);
            Elem<T>::store(orow + n, v);
        }
    }
}

int launch_gemm_simple(const GemmArgs& a, hipStream_t s) {
    if (a.max_rows <= 0 || a.G <= 0) return MOE_OK;
    const dim3 grid((a.N + kSTile - 1) / kSTile, (a.max_rows + kSTile - 1) / kSTile, a.G);
    if (a.dtype == MOE_F32)
        hipLaunchKernelGGL((gemm_simple_kernel<float>), grid, dim3(256), 0, s, a);
    else
        hipLaunchKernelGGL((gemm_simple_kernel<uint16_t>), grid, dim3(256), 0, s, a);
    return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_HIP;
}

}  // namespace moe
