// One-time re-tiling of K-major bf16 weights [G, K, N] into the operand order of the matrix cores, so that the
// GEMM kernels need no transposition on the way: inference weights are fixed, and the expert GEMMs read them at
// every call (paper Sec. 5.1: at inference the parameters' trip from memory is what costs).
//
// A work-group moves one 32 x 128 block (8 KB): rows come in with 16-byte loads (256 contiguous bytes per k-row),
// pass through LDS, and leave as eight 1 KB fragments, each lane's 16 bytes holding 8 consecutive k of one column.
#include "moe_internal.h"

namespace moe {

__global__ __launch_bounds__(256) void pack_weights_kernel(const uint16_t* __restrict__ W, uint16_t* __restrict__ P,
                                                           int K, int N, int KB, int NG) {
    __shared__ uint16_t tile[32][128 + 8];                      // +8: k-rows start 4 banks apart
    const int tid = threadIdx.x;
    const long long blk = blockIdx.x;                           // ((g*KB + kb)*NG + grp)
    const int grp = (int)(blk % NG), kb = (int)((blk / NG) % KB);
    const long long g = blk / ((long long)NG * KB);
    const uint16_t* src = W + (size_t)g * K * N;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int kr = tid / 16 + 16 * i, cp = tid % 16;
        const int k = kb * 32 + kr, n = grp * 128 + cp * 8;
        uint4 v = make_uint4(0, 0, 0, 0);
        if (k < K && n < N) v = *reinterpret_cast<const uint4*>(src + (size_t)k * N + n);
        *reinterpret_cast<uint4*>(&tile[kr][cp * 8]) = v;
    }
    __syncthreads();
    uint16_t* dst = P + (size_t)blk * 4096;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int piece = tid + 256 * i;                        // j*64 + lane
        const int j = piece / 64, lane = piece % 64, c = lane % 16, kg = lane / 16;
        uint16_t v[8];
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) v[kk] = tile[kg * 8 + kk][c * 8 + j];
        uint4 o;
        o.x = v[0] | ((uint32_t)v[1] << 16); o.y = v[2] | ((uint32_t)v[3] << 16);
        o.z = v[4] | ((uint32_t)v[5] << 16); o.w = v[6] | ((uint32_t)v[7] << 16);
        *reinterpret_cast<uint4*>(dst + (size_t)piece * 8) = o;
    }
}

int launch_pack_weights(const uint16_t* W, uint16_t* packed, int G, int K, int N, hipStream_t s) {
    const int KB = (K + 31) / 32, NG = (N + 127) / 128;
    const long long blocks = (long long)G * KB * NG;
    if (blocks <= 0) return MOE_OK;
    if (blocks >= (1ll << 31)) return MOE_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(pack_weights_kernel, dim3((unsigned)blocks), dim3(256), 0, s, W, packed, K, N, KB, NG);
    return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_HIP;
}

}  // namespace moe
