// The two data-layout transforms of paper Sec. 5.4, which take the place of the
// sparse one-hot einsums: dispatch (sort token rows by assigned expert, cost
// S x M x c_e instead of S x E x M x c_e) and combine (scale by the gate
// probability and restore token order).  Both are pure HBM-bound row moves:
// one 64-lane wave per row, 16-byte accesses, no LDS.
#include "moe_internal.h"

namespace moe {

// xe[e,c,:] = x[slot_token[e,c],:] for c < expert_rows[e].  Rows are copied as raw 16-byte words.
__global__ __launch_bounds__(256) void dispatch_kernel(const uint4* __restrict__ x, const int32_t* __restrict__ slot_token,
                                                       const int32_t* __restrict__ expert_rows, uint4* __restrict__ xe,
                                                       int E, int C, int row_vecs) {
    const int lane = threadIdx.x % kWave;
    const long long row = (long long)blockIdx.x * (blockDim.x / kWave) + threadIdx.x / kWave;
    if (row >= (long long)E * C) return;
    const int e = (int)(row / C), c = (int)(row % C);
    if (c >= expert_rows[e]) return;
    const int t = slot_token[row];
    if (t < 0) return;
    const uint4* src = x + (size_t)t * row_vecs;
    uint4* dst = xe + (size_t)row * row_vecs;
    for (int i = lane; i < row_vecs; i += kWave) dst[i] = src[i];
}

int launch_dispatch(const void* x, int dtype, const int32_t* slot_token, const int32_t* expert_rows, void* xe, int E,
                    int C, int d, hipStream_t s) {
    const int row_vecs = d * (dtype == MOE_F32 ? 4 : 2) / 16;
    const long long rows = (long long)E * C;
    const int rpb = 256 / kWave;
    hipLaunchKernelGGL(dispatch_kernel, dim3((unsigned)((rows + rpb - 1) / rpb)), dim3(256), 0, s,
                       static_cast<const uint4*>(x), slot_token, expert_rows, static_cast<uint4*>(xe), E, C, row_vecs);
    return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_HIP;
}

// out[t,:] = addend[t,:] + sum_j keep_j g_j ye[e_j, slot_j, :]   (fp32 math)
template <int K>
__global__ __launch_bounds__(256) void combine_f32_kernel(const float4* __restrict__ ye, const int32_t* __restrict__ expert_idx,
                                                          const int32_t* __restrict__ slot_idx, const float* __restrict__ gate_w,
                                                          const float4* __restrict__ addend, float4* __restrict__ out, int T,
                                                          int C, int row_vecs) {
    const int lane = threadIdx.x % kWave;
    const int t = blockIdx.x * (blockDim.x / kWave) + threadIdx.x / kWave;
    if (t >= T) return;
    const float4* src[K];
    float g[K];
#pragma unroll
    for (int j = 0; j < K; ++j) {
        const int s = slot_idx[(size_t)t * K + j];
        const int e = expert_idx[(size_t)t * K + j];
        g[j] = gate_w[(size_t)t * K + j];
        src[j] = s >= 0 ? ye + ((size_t)e * C + s) * row_vecs : nullptr;
    }
    for (int i = lane; i < row_vecs; i += kWave) {
        float4 acc = addend ? addend[(size_t)t * row_vecs + i] : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
        for (int j = 0; j < K; ++j) {
            if (src[j]) {
                const float4 v = src[j][i];
                acc.x = fmaf(g[j], v.x, acc.x);
                acc.y = fmaf(g[j], v.y, acc.y);
                acc.z = fmaf(g[j], v.z, acc.z);
                acc.w = fmaf(g[j], v.w, acc.w);
            }
        }
        out[(size_t)t * row_vecs + i] = acc;
    }
}

__device__ __forceinline__ void unpack8(const uint4& v, float* f) {
    f[0] = __uint_as_float(v.x << 16); f[1] = __uint_as_float(v.x & 0xffff0000u);
    f[2] = __uint_as_float(v.y << 16); f[3] = __uint_as_float(v.y & 0xffff0000u);
    f[4] = __uint_as_float(v.z << 16); f[5] = __uint_as_float(v.z & 0xffff0000u);
    f[6] = __uint_as_float(v.w << 16); f[7] = __uint_as_float(v.w & 0xffff0000u);
}

template <int K>
__global__ __launch_bounds__(256) void combine_bf16_kernel(const uint4* __restrict__ ye, const int32_t* __restrict__ expert_idx,
                                                           const int32_t* __restrict__ slot_idx, const float* __restrict__ gate_w,
                                                           const uint4* __restrict__ addend, uint4* __restrict__ out, int T,
                                                           int C, int row_vecs) {
    const int lane = threadIdx.x % kWave;
    const int t = blockIdx.x * (blockDim.x / kWave) + threadIdx.x / kWave;
    if (t >= T) return;
    const uint4* src[K];
    float g[K];
#pragma unroll
    for (int j = 0; j < K; ++j) {
        const int s = slot_idx[(size_t)t * K + j];
        const int e = expert_idx[(size_t)t * K + j];
        g[j] = gate_w[(size_t)t * K + j];
        src[j] = s >= 0 ? ye + ((size_t)e * C + s) * row_vecs : nullptr;
    }
    for (int i = lane; i < row_vecs; i += kWave) {
        float acc[8];
        if (addend) {
            unpack8(addend[(size_t)t * row_vecs + i], acc);
        } else {
#pragma unroll
            for (int q = 0; q < 8; ++q) acc[q] = 0.f;
        }
#pragma unroll
        for (int j = 0; j < K; ++j) {
            if (src[j]) {
                float v[8];
                unpack8(src[j][i], v);
#pragma unroll
                for (int q = 0; q < 8; ++q) acc[q] = fmaf(g[j], v[q], acc[q]);
            }
        }
        uint4 o;
        o.x = pack_bf16x2(acc[0], acc[1]);
        o.y = pack_bf16x2(acc[2], acc[3]);
        o.z = pack_bf16x2(acc[4], acc[5]);
        o.w = pack_bf16x2(acc[6], acc[7]);
        out[(size_t)t * row_vecs + i] = o;
    }
}

int launch_combine(const void* ye, int dtype, const int32_t* expert_idx, const int32_t* slot_idx, const float* gate_w,
                   const void* addend, void* out, int T, int k, int C, int d, hipStream_t s) {
    const int rpb = 256 / kWave;
    const dim3 grid((T + rpb - 1) / rpb), block(256);
    if (dtype == MOE_F32) {
        const int rv = d / 4;
        if (k == 1)
            hipLaunchKernelGGL((combine_f32_kernel<1>), grid, block, 0, s, static_cast<const float4*>(ye), expert_idx,
                               slot_idx, gate_w, static_cast<const float4*>(addend), static_cast<float4*>(out), T, C, rv);
        else
            hipLaunchKernelGGL((combine_f32_kernel<2>), grid, block, 0, s, static_cast<const float4*>(ye), expert_idx,
                               slot_idx, gate_w, static_cast<const float4*>(addend), static_cast<float4*>(out), T, C, rv);
    } else {
        const int rv = d / 8;
        if (k == 1)
            hipLaunchKernelGGL((combine_bf16_kernel<1>), grid, block, 0, s, static_cast<const uint4*>(ye), expert_idx,
                               slot_idx, gate_w, static_cast<const uint4*>(addend), static_cast<uint4*>(out), T, C, rv);
        else
            hipLaunchKernelGGL((combine_bf16_kernel<2>), grid, block, 0, s, static_cast<const uint4*>(ye), expert_idx,
                               slot_idx, gate_w, static_cast<const uint4*>(addend), static_cast<uint4*>(out), T, C, rv);
    }
    return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_HIP;
}

}  // namespace moe
