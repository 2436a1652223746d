// The non-expert half of a decoder block for one decode step (one new token per sequence): LayerNorm, attention of
// the new token over its sequence's key/value cache, residual adds.  The paper runs such kernels beside the MoE
// kernels (Sec. 5.4, first paragraph; model shapes in Sec. 3.1) and gives no design for them; everything here is
// bound by memory traffic (the cache is read once per step), so the kernels are plain 16-byte streaming loops.
#include "moe_internal.h"

namespace moe {

__device__ __forceinline__ void unpack8(const uint4 v, float (&f)[8]) {
    f[0] = __uint_as_float(v.x << 16); f[1] = __uint_as_float(v.x & 0xffff0000u);
    f[2] = __uint_as_float(v.y << 16); f[3] = __uint_as_float(v.y & 0xffff0000u);
    f[4] = __uint_as_float(v.z << 16); f[5] = __uint_as_float(v.z & 0xffff0000u);
    f[6] = __uint_as_float(v.w << 16); f[7] = __uint_as_float(v.w & 0xffff0000u);
}
__device__ __forceinline__ uint4 pack8(const float (&f)[8]) {
    return make_uint4(pack_bf16x2(f[0], f[1]), pack_bf16x2(f[2], f[3]), pack_bf16x2(f[4], f[5]), pack_bf16x2(f[6], f[7]));
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m);
    return v;
}

// y[t,:] = LayerNorm(s[t,:]) * gamma + beta with s = x (+ r), one wave per row; s is also written to `sum_out` when
// given (rounded to bf16 first: the statistics are those of the stored row).  d is a multiple of 8.
__global__ __launch_bounds__(256) void add_layernorm_kernel(const uint16_t* __restrict__ x, const uint16_t* __restrict__ r,
                                                            const float* __restrict__ gamma, const float* __restrict__ beta,
                                                            uint16_t* __restrict__ sum_out, uint16_t* __restrict__ y, int T,
                                                            int d, float eps) {
    const int lane = threadIdx.x & 63;
    const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (t >= T) return;
    const int pieces = d / 8;
    const uint4* xr = reinterpret_cast<const uint4*>(x + (size_t)t * d);
    const uint4* rr = r ? reinterpret_cast<const uint4*>(r + (size_t)t * d) : nullptr;
    auto row_piece = [&](int i, float (&f)[8]) {
        unpack8(xr[i], f);
        if (rr) {
            float g[8];
            unpack8(rr[i], g);
#pragma unroll
            for (int q = 0; q < 8; ++q) f[q] += g[q];
            unpack8(pack8(f), f);                       // the row as it is stored
        }
    };
    float sum = 0.f;
    for (int i = lane; i < pieces; i += 64) {
        float f[8];
        row_piece(i, f);
        if (sum_out) reinterpret_cast<uint4*>(sum_out + (size_t)t * d)[i] = pack8(f);
#pragma unroll
        for (int q = 0; q < 8; ++q) sum += f[q];
    }
    const float mean = wave_sum(sum) / (float)d;
    float sq = 0.f;
    for (int i = lane; i < pieces; i += 64) {
        float f[8];
        row_piece(i, f);
#pragma unroll
        for (int q = 0; q < 8; ++q) sq += (f[q] - mean) * (f[q] - mean);
    }
    const float rstd = rsqrtf(wave_sum(sq) / (float)d + eps);
    for (int i = lane; i < pieces; i += 64) {
        float f[8];
        row_piece(i, f);
        const float4 g0 = reinterpret_cast<const float4*>(gamma)[2 * i], g1 = reinterpret_cast<const float4*>(gamma)[2 * i + 1];
        const float4 b0 = reinterpret_cast<const float4*>(beta)[2 * i], b1 = reinterpret_cast<const float4*>(beta)[2 * i + 1];
        const float g[8] = {g0.x, g0.y, g0.z, g0.w, g1.x, g1.y, g1.z, g1.w};
        const float b[8] = {b0.x, b0.y, b0.z, b0.w, b1.x, b1.y, b1.z, b1.w};
#pragma unroll
        for (int q = 0; q < 8; ++q) f[q] = (f[q] - mean) * rstd * g[q] + b[q];
        reinterpret_cast<uint4*>(y + (size_t)t * d)[i] = pack8(f);
    }
}

int launch_add_layernorm(const uint16_t* x, const uint16_t* r, const float* gamma, const float* beta, uint16_t* sum_out,
                         uint16_t* y, int T, int d, float eps, hipStream_t s) {
    hipLaunchKernelGGL(add_layernorm_kernel, dim3((T + 3) / 4), dim3(256), 0, s, x, r, gamma, beta, sum_out, y, T, d, eps);
    return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_HIP;
}

// out = a + b, bf16, n8 pieces of 8 elements
__global__ __launch_bounds__(256) void add_rows_kernel(const uint4* __restrict__ a, const uint4* __restrict__ b,
                                                       uint4* __restrict__ out, long long n8) {
    for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < n8; i += (long long)gridDim.x * 256) {
        float f[8], g[8];
        unpack8(a[i], f);
        unpack8(b[i], g);
#pragma unroll
        for (int q = 0; q < 8; ++q) f[q] += g[q];
        out[i] = pack8(f);
    }
}
int launch_add_rows(const uint16_t* a, const uint16_t* b, uint16_t* out, long long n, hipStream_t s) {
    const long long n8 = n / 8;
    long long blocks = (n8 + 255) / 256;
    if (blocks > 2048) blocks = 2048;
    hipLaunchKernelGGL(add_rows_kernel, dim3((unsigned)blocks), dim3(256), 0, s, reinterpret_cast<const uint4*>(a),
                       reinterpret_cast<const uint4*>(b), reinterpret_cast<uint4*>(out), n8);
    return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_HIP;
}

// ---- attention of one new token per sequence over its cache ---------------------------------------------------
// qkv [T, 3d] holds the new token's query, key and value (head h: columns h*DH.. of each third); the caches are
// [T, H, Lmax, DH]; sequence b has pos[b] cached positions and the new token is position pos[b].
// A work-group takes kAttnChunk consecutive positions of one (sequence, head); LPP = DH/8 lanes share a position
// (16 bytes of its key and value each), a wave step covers 64/LPP consecutive positions = 1 KB of contiguous cache.
// Every lane group keeps a running softmax (maximum, sum, weighted values); the groups of a work-group meet in LDS
// and leave one partial (m, l, o[DH]) per chunk, merged by attn_merge_kernel.  The chunk that holds position pos[b]
// takes the new key/value from qkv, never from the cache, so the write of the new rows into the cache (by chunk 0)
// races with nobody.
constexpr int kAttnChunk = 256;

template <int DH>
__global__ __launch_bounds__(256) void attn_decode_kernel(const uint16_t* __restrict__ qkv, uint16_t* __restrict__ cache_k,
                                                          uint16_t* __restrict__ cache_v, const int32_t* __restrict__ pos,
                                                          float* __restrict__ partial, int H, int Lmax, int nsplit) {
    constexpr int LPP = DH / 8, PPW = 64 / LPP, NG = 4 * PPW;       // lanes per position, positions per wave step, groups
    __shared__ float m_sh[NG], l_sh[NG];
    __shared__ float o_sh[NG][DH];
    const int bh = blockIdx.x, b = bh / H, h = bh % H, split = blockIdx.y;
    const int d = H * DH;
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int sub = lane % LPP, grp = lane / LPP;
    const int npast = min(max(pos[b], 0), Lmax - 1);                 // cached positions (clamped into the cache: no
                                                                     // access can leave it); the new token is position npast
    const uint16_t* qrow = qkv + (size_t)b * 3 * d + h * DH;
    float q[8];
    unpack8(*reinterpret_cast<const uint4*>(qrow + sub * 8), q);
    const float scale = rsqrtf((float)DH);
#pragma unroll
    for (int i = 0; i < 8; ++i) q[i] *= scale;
    const uint16_t* kc = cache_k + ((size_t)b * H + h) * Lmax * DH;
    const uint16_t* vc = cache_v + ((size_t)b * H + h) * Lmax * DH;
    if (split == 0 && tid < 2 * LPP) {                               // the new rows join the cache for later steps
        const int which = tid / LPP, piece = tid % LPP;
        const uint4 v = *reinterpret_cast<const uint4*>(qrow + (1 + which) * d + piece * 8);
        uint16_t* dst = (which ? cache_v : cache_k) + (((size_t)b * H + h) * Lmax + npast) * DH + piece * 8;
        *reinterpret_cast<uint4*>(dst) = v;
    }
    float m = -INFINITY, l = 0.f, o[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) o[i] = 0.f;
    const int p0 = split * kAttnChunk + w * (kAttnChunk / 4);
    for (int step = 0; step < kAttnChunk / 4 / PPW; ++step) {
        const int p = p0 + step * PPW + grp;
        if (p0 + step * PPW > npast) break;                          // uniform over the wave
        const bool valid = p <= npast;
        const int pc = min(p, max(npast - 1, 0));                    // clamped cache position (in bounds; unused if !valid)
        uint4 kraw = *reinterpret_cast<const uint4*>(kc + (size_t)pc * DH + sub * 8);
        uint4 vraw = *reinterpret_cast<const uint4*>(vc + (size_t)pc * DH + sub * 8);
        if (p == npast || npast == 0) {                              // the new token itself
            kraw = *reinterpret_cast<const uint4*>(qrow + d + sub * 8);
            vraw = *reinterpret_cast<const uint4*>(qrow + 2 * d + sub * 8);
        }
        float kf[8], vf[8];
        unpack8(kraw, kf);
        unpack8(vraw, vf);
        float s = 0.f;
#pragma unroll
        for (int i = 0; i < 8; ++i) s = fmaf(q[i], kf[i], s);
#pragma unroll
        for (int msk = 1; msk < LPP; msk <<= 1) s += __shfl_xor(s, msk);
        if (valid) {
            const float mn = fmaxf(m, s);
            const float c = __expf(m - mn), e = __expf(s - mn);      // m = -inf at first: c = 0
            l = l * c + e;
#pragma unroll
            for (int i = 0; i < 8; ++i) o[i] = fmaf(o[i], c, e * vf[i]);
            m = mn;
        }
    }
    const int g = w * PPW + grp;
    if (sub == 0) { m_sh[g] = m; l_sh[g] = l; }
#pragma unroll
    for (int i = 0; i < 8; ++i) o_sh[g][sub * 8 + i] = o[i];
    __syncthreads();
    if (tid < DH) {
        float M = -INFINITY;
        for (int j = 0; j < NG; ++j) M = fmaxf(M, m_sh[j]);
        float L = 0.f, O = 0.f;
        if (M > -INFINITY) {
            for (int j = 0; j < NG; ++j) {
                const float c = __expf(m_sh[j] - M);                 // empty groups: exp(-inf) = 0
                L = fmaf(l_sh[j], c, L);
                O = fmaf(o_sh[j][tid], c, O);
            }
        }
        float* dst = partial + ((size_t)bh * nsplit + split) * (DH + 2);
        dst[2 + tid] = O;
        if (tid == 0) { dst[0] = M; dst[1] = L; }
    }
}

// attn[b, h*DH + t] = sum_split o * exp(m - M) / sum_split l * exp(m - M)
template <int DH>
__global__ __launch_bounds__(DH) void attn_merge_kernel(const float* __restrict__ partial, uint16_t* __restrict__ attn, int H,
                                                        int nsplit) {
    const int bh = blockIdx.x, b = bh / H, h = bh % H, t = threadIdx.x;
    const float* p = partial + (size_t)bh * nsplit * (DH + 2);
    float M = -INFINITY;
    for (int s = 0; s < nsplit; ++s) M = fmaxf(M, p[s * (DH + 2)]);
    float L = 0.f, O = 0.f;
    for (int s = 0; s < nsplit; ++s) {
        const float c = __expf(p[s * (DH + 2)] - M);
        L = fmaf(p[s * (DH + 2) + 1], c, L);
        O = fmaf(p[s * (DH + 2) + 2 + t], c, O);
    }
    attn[(size_t)b * H * DH + h * DH + t] = f32_to_bf16(O / L);
}

int attn_nsplit(int Lmax) { return (Lmax + kAttnChunk - 1) / kAttnChunk; }
size_t attn_partial_floats(int T, int H, int dh, int Lmax) { return (size_t)T * H * attn_nsplit(Lmax) * (dh + 2); }
bool attn_supported(int d, int H) { return H >= 1 && d % H == 0 && (d / H == 64 || d / H == 128); }

int launch_attn_decode(const uint16_t* qkv, uint16_t* cache_k, uint16_t* cache_v, const int32_t* pos, float* partial,
                       uint16_t* attn, int T, int H, int dh, int Lmax, hipStream_t s) {
    const int nsplit = attn_nsplit(Lmax);
    const dim3 grid((unsigned)(T * H), (unsigned)nsplit);
    if (dh == 128) {
        hipLaunchKernelGGL((attn_decode_kernel<128>), grid, dim3(256), 0, s, qkv, cache_k, cache_v, pos, partial, H, Lmax, nsplit);
        hipLaunchKernelGGL((attn_merge_kernel<128>), dim3((unsigned)(T * H)), dim3(128), 0, s, partial, attn, H, nsplit);
    } else {
        hipLaunchKernelGGL((attn_decode_kernel<64>), grid, dim3(256), 0, s, qkv, cache_k, cache_v, pos, partial, H, Lmax, nsplit);
        hipLaunchKernelGGL((attn_merge_kernel<64>), dim3((unsigned)(T * H)), dim3(64), 0, s, partial, attn, H, nsplit);
    }
    return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_HIP;
}

}  // namespace moe
