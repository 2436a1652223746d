// Stand-alone measurement: what a kernel that does nothing but read reaches on this chip, with the access
// patterns of the weight-streaming expert GEMM.  It is the practical ceiling for that kernel's HBM rate.
//
//     paper_2201_05596_amd/hbm_rate
//
// "linear": every wave reads one contiguous slab with 16-byte loads, 8 or 16 in flight, plain or with the
// non-temporal hint.  "strips": a [G][K][N] array of 2-byte weights; a wave reads a strip of 128 columns
// (256 bytes per row, 4 rows per load instruction) down all K rows, non-temporal, 8 loads in flight; either
// waves dealt to the XCDs in launch order, or work-groups of two waves with all strips of a matrix on one XCD
// (as the GEMM deals its tiles), or 256 resident work-groups of four waves that walk their XCD's strips (the
// occupancy of the 64-row GEMM kernels: one wave per SIMD).
#include <hip/hip_runtime.h>
#include <cstdint>
#include <cstdio>

typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));

#define CHECK(x)                                                                   \
    do {                                                                           \
        hipError_t e_ = (x);                                                       \
        if (e_ != hipSuccess) {                                                    \
            fprintf(stderr, "%s failed: %s\n", #x, hipGetErrorString(e_));         \
            return 1;                                                              \
        }                                                                          \
    } while (0)

__device__ __forceinline__ void consume(const u32x4_t& acc, u32x4_t* sink) {
    if (acc.x == 0x12345678u && acc.y == 0x9abcdef0u) sink[0] = acc;      // never true for the fill pattern
}

template <int U, bool NT>
__global__ __launch_bounds__(256) void read_linear(const u32x4_t* __restrict__ p, size_t per_wave, u32x4_t* sink) {
    const int lane = threadIdx.x & 63;
    const size_t wave = (size_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const u32x4_t* q = p + wave * per_wave + lane;
    u32x4_t acc = {0, 0, 0, 0};
    for (size_t i = 0; i + 64 * U <= per_wave; i += 64 * U) {
        u32x4_t v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) v[u] = NT ? __builtin_nontemporal_load(q + i + u * 64) : q[i + u * 64];
#pragma unroll
        for (int u = 0; u < U; ++u) acc ^= v[u];
    }
    consume(acc, sink);
}

template <bool PER_XCD>
__global__ __launch_bounds__(256) void read_strips(const char* __restrict__ p, int G, int K, int N, u32x4_t* sink) {
    constexpr int U = 8;
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int strips = N / 128;
    int g, st;
    if (PER_XCD) {                      // blockDim.x == 128: two strips per work-group, matrix g on XCD g % 8
        const int xcd = blockIdx.x % 8, q = blockIdx.x / 8, per_g = strips / 2;
        g = (q / per_g) * 8 + xcd;
        st = (q % per_g) * 2 + w;
    } else {
        const size_t wave = (size_t)blockIdx.x * 4 + w;
        g = (int)(wave / strips);
        st = (int)(wave % strips);
    }
    if (g >= G) return;
    const char* q = p + (size_t)g * K * N * 2 + (size_t)(lane >> 4) * N * 2 + st * 256 + (lane & 15) * 16;
    u32x4_t acc = {0, 0, 0, 0};
    for (int k = 0; k + 4 * U <= K; k += 4 * U) {
        u32x4_t v[U];
#pragma unroll
        for (int u = 0; u < U; ++u)
            v[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(q + (size_t)(k + 4 * u) * N * 2));
#pragma unroll
        for (int u = 0; u < U; ++u) acc ^= v[u];
    }
    consume(acc, sink);
}

// As read_strips<true>, but with the occupancy the MT = 64 GEMM kernels have: one work-group of 4 waves per CU
// (one wave per SIMD), each wave walking the strips w, w + 1024, ... of its XCD's matrices.
__global__ __launch_bounds__(256) void read_strips_resident(const char* __restrict__ p, int G, int K, int N, u32x4_t* sink) {
    constexpr int U = 8;
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int xcd = blockIdx.x % 8, per_g = N / 512;                 // work-group tiles of 4 strips per matrix
    const int groups_per_xcd = (G + 7) / 8;
    u32x4_t acc = {0, 0, 0, 0};
    for (int q = blockIdx.x / 8; q < groups_per_xcd * per_g; q += gridDim.x / 8) {
        const int g = (q / per_g) * 8 + xcd, st = (q % per_g) * 4 + w;
        if (g >= G) continue;
        const char* base = p + (size_t)g * K * N * 2 + (size_t)(lane >> 4) * N * 2 + st * 256 + (lane & 15) * 16;
        for (int k = 0; k + 4 * U <= K; k += 4 * U) {
            u32x4_t v[U];
#pragma unroll
            for (int u = 0; u < U; ++u)
                v[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(base + (size_t)(k + 4 * u) * N * 2));
#pragma unroll
            for (int u = 0; u < U; ++u) acc ^= v[u];
        }
    }
    consume(acc, sink);
}

template <class F> static float best_ms(F launch) {
    hipEvent_t e0, e1;
    (void)hipEventCreate(&e0);
    (void)hipEventCreate(&e1);
    launch();
    float best = 1e30f;
    for (int rep = 0; rep < 3; ++rep) {
        (void)hipEventRecord(e0, 0);
        launch();
        (void)hipEventRecord(e1, 0);
        (void)hipEventSynchronize(e1);
        float ms = 0.f;
        (void)hipEventElapsedTime(&ms, e0, e1);
        best = ms < best ? ms : best;
    }
    return best;
}

int main() {
    const size_t bytes = 1ull << 30;
    char* p;
    u32x4_t* sink;
    CHECK(hipMalloc(&p, bytes));
    CHECK(hipMemset(p, 1, bytes));
    CHECK(hipMalloc(&sink, 64));
    const u32x4_t* pv = reinterpret_cast<const u32x4_t*>(p);
    for (int blocks : {1024, 4096}) {
        const size_t per_wave = bytes / 16 / ((size_t)blocks * 4);
        const float t0 = best_ms([&] { hipLaunchKernelGGL((read_linear<8, false>), dim3(blocks), dim3(256), 0, 0, pv, per_wave, sink); });
        const float t1 = best_ms([&] { hipLaunchKernelGGL((read_linear<8, true>), dim3(blocks), dim3(256), 0, 0, pv, per_wave, sink); });
        const float t2 = best_ms([&] { hipLaunchKernelGGL((read_linear<16, true>), dim3(blocks), dim3(256), 0, 0, pv, per_wave, sink); });
        printf("{\"pattern\": \"linear\", \"MiB\": 1024, \"work_groups\": %d, \"plain_8_TBps\": %.2f, \"nontemporal_8_TBps\": %.2f, "
               "\"nontemporal_16_TBps\": %.2f}\n", blocks, bytes / (t0 * 1e9), bytes / (t1 * 1e9), bytes / (t2 * 1e9));
    }
    const struct { const char* name; int G, K, N; } shapes[] = {
        {"c2 W1", 128, 1024, 4096}, {"c2 W2", 128, 4096, 1024}, {"c4 W1 (32 experts)", 32, 2048, 8192}, {"c4 W2 (32 experts)", 32, 8192, 2048}};
    for (const auto& s : shapes) {
        const size_t total = (size_t)s.G * s.K * s.N * 2;
        if (total > bytes || s.N % 256 != 0 || s.K % 32 != 0) return 3;
        const size_t waves = (size_t)s.G * (s.N / 128);
        const int b1 = (int)((waves + 3) / 4), b2 = (s.G + 7) / 8 * 8 * (s.N / 256);
        const float t1 = best_ms([&] { hipLaunchKernelGGL((read_strips<false>), dim3(b1), dim3(256), 0, 0, p, s.G, s.K, s.N, sink); });
        const float t2 = best_ms([&] { hipLaunchKernelGGL((read_strips<true>), dim3(b2), dim3(128), 0, 0, p, s.G, s.K, s.N, sink); });
        const float t3 = s.N % 512 ? 0.f : best_ms([&] { hipLaunchKernelGGL(read_strips_resident, dim3(256), dim3(256), 0, 0, p, s.G, s.K, s.N, sink); });
        printf("{\"pattern\": \"strips\", \"weights\": \"%s\", \"G\": %d, \"K\": %d, \"N\": %d, \"MiB\": %zu, \"waves\": %zu, "
               "\"launch_order_TBps\": %.2f, \"matrix_per_xcd_TBps\": %.2f, \"one_wave_per_simd_TBps\": %.2f}\n", s.name, s.G, s.K, s.N,
               total >> 20, waves, total / (t1 * 1e9), total / (t2 * 1e9), t3 > 0.f ? total / (t3 * 1e9) : 0.0);
    }
    CHECK(hipGetLastError());
    return 0;
}
