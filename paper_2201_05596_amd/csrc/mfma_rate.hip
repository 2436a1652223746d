// Stand-alone measurement: the rate at which the chip sustains v_mfma_f32_16x16x32_bf16 when nothing else
// happens (no memory traffic, no LDS, no barriers), with operands of zeros and with random bf16 operands.
// It is the practical ceiling for the tiled expert GEMM (the kernel for experts with many tokens): the
// sustained matrix rate depends on the operand data.
//
//     paper_2201_05596_amd/mfma_rate [iterations]
//
// Every CU gets one work-group of 8 waves (two per SIMD, as in the tiled kernel); a wave keeps a 64 x 128
// accumulator tile (32 MFMA destinations) and cycles through 4 + 8 operand fragments held in registers.
#include <hip/hip_runtime.h>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

#define CHECK(x)                                                                              \
    do {                                                                                      \
        hipError_t e_ = (x);                                                                  \
        if (e_ != hipSuccess) {                                                               \
            fprintf(stderr, "%s failed: %s\n", #x, hipGetErrorString(e_));                    \
            return 1;                                                                         \
        }                                                                                     \
    } while (0)

__global__ __launch_bounds__(512) void mfma_rate_kernel(const uint4* __restrict__ operands, float* __restrict__ sink,
                                                        int iterations) {
    const int lane_id = blockIdx.x * 512 + threadIdx.x;
    bf16x8_t a[4], b[8];
#pragma unroll
    for (int i = 0; i < 4; ++i) a[i] = __builtin_bit_cast(bf16x8_t, operands[(size_t)lane_id * 12 + i]);
#pragma unroll
    for (int j = 0; j < 8; ++j) b[j] = __builtin_bit_cast(bf16x8_t, operands[(size_t)lane_id * 12 + 4 + j]);
    f32x4_t acc[4][8];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[i][j] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    for (int it = 0; it < iterations; ++it) {
#pragma unroll
        for (int j = 0; j < 8; ++j)
#pragma unroll
            for (int i = 0; i < 4; ++i) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j) s += acc[i][j][0] + acc[i][j][1] + acc[i][j][2] + acc[i][j][3];
    sink[lane_id] = s;
}

int main(int argc, char** argv) {
    const int iterations = argc > 1 ? atoi(argv[1]) : 20000;
    if (iterations <= 0 || iterations > 1000000) {
        fprintf(stderr, "iterations must be in 1..1000000\n");
        return 2;
    }
    hipDeviceProp_t prop;
    CHECK(hipGetDeviceProperties(&prop, 0));
    const int blocks = prop.multiProcessorCount;
    const size_t lanes = (size_t)blocks * 512;
    uint4* operands;
    float* sink;
    CHECK(hipMalloc(&operands, lanes * 12 * sizeof(uint4)));
    CHECK(hipMalloc(&sink, lanes * sizeof(float)));
    hipEvent_t e0, e1;
    CHECK(hipEventCreate(&e0));
    CHECK(hipEventCreate(&e1));
    const double flops = (double)blocks * 8 * iterations * 32 * (2.0 * 16 * 16 * 32);
    for (int random_data = 0; random_data < 2; ++random_data) {
        std::vector<uint16_t> h(lanes * 12 * 8, 0);
        if (random_data) {                       // bf16 values of either sign between about 0.01 and 2
            uint32_t st = 12345u;
            for (auto& v : h) {
                st = st * 1664525u + 1013904223u;
                v = (uint16_t)(((st >> 16) & 0x807f) | 0x3c00 | ((st >> 9) & 0x0380));
            }
        }
        CHECK(hipMemcpy(operands, h.data(), h.size() * 2, hipMemcpyHostToDevice));
        hipLaunchKernelGGL(mfma_rate_kernel, dim3(blocks), dim3(512), 0, 0, operands, sink, 100);   // warm-up
        float best = 1e30f;
        for (int rep = 0; rep < 3; ++rep) {
            CHECK(hipEventRecord(e0, 0));
            hipLaunchKernelGGL(mfma_rate_kernel, dim3(blocks), dim3(512), 0, 0, operands, sink, iterations);
            CHECK(hipEventRecord(e1, 0));
            CHECK(hipEventSynchronize(e1));
            float ms;
            CHECK(hipEventElapsedTime(&ms, e0, e1));
            best = ms < best ? ms : best;
        }
        CHECK(hipGetLastError());
        printf("{\"operands\": \"%s\", \"CUs\": %d, \"ms\": %.3f, \"TFLOPs\": %.1f, \"frac_of_2500\": %.3f}\n",
               random_data ? "random bf16" : "zeros", blocks, best, flops / (best * 1e-3) / 1e12, flops / (best * 1e-3) / 2.5e15);
    }
    return 0;
}
