// MFMA-only rate of this machine: a register-only loop of v_mfma_f32_32x32x16_bf16 (no memory traffic, no LDS,
// no vector work), 8 independent accumulators, 2 wavefronts per SIMD on all 256 CUs.  Stand-alone program that
// bench.py runs as a child process to report what the matrix cores sustain next to the nominal peak:
//     hipcc --offload-arch=gfx950 -O3 -o mfma_peak mfma_peak.hip && ./mfma_peak
// prints two figures in TFLOP/s: constant operands (best of 5 launches), and operands that differ from one
// MFMA to the next (pseudo-random bf16 in [-2, 2), launches of about 50 ms so that the clock settles).
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

#define CHECK(x)                                                                      \
    do {                                                                              \
        hipError_t e_ = (x);                                                          \
        if (e_ != hipSuccess) { printf("HIP error %s at %s:%d\n", hipGetErrorString(e_), __FILE__, __LINE__); exit(1); } \
    } while (0)

__global__ __launch_bounds__(256) void mfma_constant_operands(float* out, int iters)
{
    bf16x8 a, b;
    for (int e = 0; e < 8; ++e) { a[e] = (__bf16)(float)(threadIdx.x % 3); b[e] = (__bf16)1.0f; }
    f32x16 c[8];
    for (int i = 0; i < 8; ++i) for (int r = 0; r < 16; ++r) c[i][r] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 8; ++i) asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(c[i]) : "v"(a), "v"(b));
    }
    float s = 0;
    for (int i = 0; i < 8; ++i) for (int r = 0; r < 16; ++r) s += c[i][r];
    if (s == 12345.f) out[0] = s;
}

__device__ inline unsigned mix32(unsigned x) { x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16; return x; }
__global__ __launch_bounds__(256) void mfma_random_operands(float* out, int iters)
{
    bf16x8 a[8], b[8];
    for (int i = 0; i < 8; ++i)
        for (int e = 0; e < 8; ++e) {
            const unsigned r = mix32(threadIdx.x * 131u + i * 17u + e * 3u + blockIdx.x * 7919u);
            a[i][e] = (__bf16)(((int)(r & 0xffff) - 32768) * (1.0f / 16384.f));
            b[i][e] = (__bf16)(((int)(r >> 16) - 32768) * (1.0f / 16384.f));
        }
    f32x16 c[8];
    for (int i = 0; i < 8; ++i) for (int r = 0; r < 16; ++r) c[i][r] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 8; ++i) asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(c[i]) : "v"(a[i]), "v"(b[i]));
        if ((it & 1023) == 1023)                       // keep the accumulators finite
            for (int i = 0; i < 8; ++i) for (int r = 0; r < 16; ++r) c[i][r] *= 1e-3f;
    }
    float s = 0;
    for (int i = 0; i < 8; ++i) for (int r = 0; r < 16; ++r) s += c[i][r];
    if (s == 12345.f) out[0] = s;
}

static float* g_f;

template <typename K>
static double tflops(K kernel, int iters)
{
    const int w = 2;                                   // wavefronts per SIMD
    hipEvent_t a, b;
    CHECK(hipEventCreate(&a));
    CHECK(hipEventCreate(&b));
    hipLaunchKernelGGL(kernel, dim3(256 * w), dim3(256), 0, 0, g_f, 100);
    CHECK(hipEventRecord(a));
    hipLaunchKernelGGL(kernel, dim3(256 * w), dim3(256), 0, 0, g_f, iters);
    CHECK(hipEventRecord(b));
    CHECK(hipEventSynchronize(b));
    float ms;
    CHECK(hipEventElapsedTime(&ms, a, b));
    CHECK(hipGetLastError());
    // work-groups x wavefronts x iterations x 8 MFMAs x 2*32*32*16 FLOP
    return 256.0 * w * 4.0 * iters * 8.0 * 32768.0 / (ms * 1e-3) / 1e12;
}

int main()
{
    CHECK(hipMalloc(&g_f, 1024));
    double best = 0.0, best_rand = 0.0;
    for (int rep = 0; rep < 5; ++rep) { const double t = tflops(mfma_constant_operands, 20000); best = t > best ? t : best; }
    for (int rep = 0; rep < 3; ++rep) { const double t = tflops(mfma_random_operands, 200000); best_rand = t > best_rand ? t : best_rand; }
    printf("%.1f %.1f\n", best, best_rand);
    return 0;
}
