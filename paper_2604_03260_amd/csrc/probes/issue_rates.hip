// Register-only issue-rate probes for gfx950 (no memory traffic, no LDS): what one SIMD sustains when the
// matrix core and the vector ALU are used together, and what the fp64 vector rate needs.  Stand-alone
// program, not part of libfocus.so:
//     hipcc --offload-arch=gfx950 -O3 -o issue_rates issue_rates.hip && ./issue_rates
// Every figure is wall time converted to cycles of the nominal 2.4 GHz clock per instruction group per SIMD
// (256 CUs x 4 SIMDs; `w` work-groups of 256 threads per CU = `w` wavefronts per SIMD).
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
#include <string>

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;

#define CHECK(x)                                                                      \
    do {                                                                              \
        hipError_t e_ = (x);                                                          \
        if (e_ != hipSuccess) { printf("HIP error %s at %s:%d\n", hipGetErrorString(e_), __FILE__, __LINE__); exit(1); } \
    } while (0)

// ---- 1. one MFMA followed by NV vector instructions, 8 independent accumulators, order fixed by inline asm
// KIND 0: v_exp_f32, 1: v_fma_f32, 2: no MFMA + v_fma_f32, 3: no MFMA + v_exp_f32.  BIG: 32x32x16, else 16x16x32.
template <int NV, int KIND, bool BIG>
__global__ __launch_bounds__(256) void mfma_valu(float* out, int iters)
{
    bf16x8 a, b;
    for (int e = 0; e < 8; ++e) { a[e] = (__bf16)(float)(threadIdx.x % 3); b[e] = (__bf16)1.0f; }
    f32x16 c[8];
    f32x4 c4[8];
    for (int i = 0; i < 8; ++i) {
        for (int r = 0; r < 16; ++r) c[i][r] = 0.f;
        for (int r = 0; r < 4; ++r) c4[i][r] = 0.f;
    }
    float x[8];
    for (int i = 0; i < 8; ++i) x[i] = 0.001f * threadIdx.x + i;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            if (KIND < 2) {
                if (BIG) asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(c[i]) : "v"(a), "v"(b));
                else asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+v"(c4[i]) : "v"(a), "v"(b));
            }
#pragma unroll
            for (int v = 0; v < NV; ++v) {
                if (KIND == 0 || KIND == 3) asm volatile("v_exp_f32 %0, %0" : "+v"(x[v % 8]));
                else asm volatile("v_fma_f32 %0, %0, %0, %0" : "+v"(x[v % 8]));
            }
        }
    }
    float s = 0;
    for (int i = 0; i < 8; ++i) { s += x[i]; for (int r = 0; r < 16; ++r) s += c[i][r]; for (int r = 0; r < 4; ++r) s += c4[i][r]; }
    if (s == 12345.f) out[0] = s;
}

// ---- 2. fp64 FMA with CH independent accumulators (second operand wave-uniform, as in the scoring kernels)
template <int CH>
__global__ __launch_bounds__(256) void fma64(double* out, const double* __restrict__ w, int iters)
{
    double a[CH];
    for (int i = 0; i < CH; ++i) a[i] = threadIdx.x * 1e-3 + i;
    const double x = 1.0 + threadIdx.x * 1e-9;
    for (int it = 0; it < iters; ++it) {
        const double* wr = w + (it & 63) * 16;
#pragma unroll
        for (int rep = 0; rep < 16 / CH; ++rep)
#pragma unroll
            for (int i = 0; i < CH; ++i) a[i] = fma(x, wr[rep * CH + i], a[i]);
    }
    double s = 0;
    for (int i = 0; i < CH; ++i) s += a[i];
    if (s == 12345.678) out[0] = s;
}

// ---- 3. fp64 MFMA 16x16x4 (1024 FMAs = 16 wave-wide FMA instructions)
__global__ __launch_bounds__(256) void mfma64(double* out, int iters)
{
    typedef double d4 __attribute__((ext_vector_type(4)));
    const double x = 1.0 + threadIdx.x * 1e-9, y = 0.999999;
    d4 c0 = {0, 0, 0, 0}, c1 = c0, c2 = c0, c3 = c0;
    for (int it = 0; it < iters; ++it) {
        c0 = __builtin_amdgcn_mfma_f64_16x16x4f64(x, y, c0, 0, 0, 0);
        c1 = __builtin_amdgcn_mfma_f64_16x16x4f64(x, y, c1, 0, 0, 0);
        c2 = __builtin_amdgcn_mfma_f64_16x16x4f64(x, y, c2, 0, 0, 0);
        c3 = __builtin_amdgcn_mfma_f64_16x16x4f64(x, y, c3, 0, 0, 0);
    }
    double s = 0;
    for (int i = 0; i < 4; ++i) s += c0[i] + c1[i] + c2[i] + c3[i];
    if (s == 12345.678) out[0] = s;
}

static float timed(void (*launch)(int grid, int iters), int grid, int iters)
{
    hipEvent_t a, b;
    CHECK(hipEventCreate(&a));
    CHECK(hipEventCreate(&b));
    launch(grid, 100);
    CHECK(hipEventRecord(a));
    launch(grid, iters);
    CHECK(hipEventRecord(b));
    CHECK(hipEventSynchronize(b));
    float ms;
    CHECK(hipEventElapsedTime(&ms, a, b));
    CHECK(hipGetLastError());
    return ms;
}

static float* g_f;
static double *g_d, *g_w;
static double cycles_per_group(float ms, int w, int iters, int groups_per_iter)
{
    return ms * 1e-3 * 2.4e9 / ((double)w * iters * groups_per_iter);
}

template <int NV, int KIND, bool BIG> void run_mv(int w)
{
    const int iters = 20000;
    const float ms = timed([](int g, int it) { hipLaunchKernelGGL((mfma_valu<NV, KIND, BIG>), dim3(g), dim3(256), 0, 0, g_f, it); },
                           256 * w, iters);
    printf("  %-9s + %2d x %-9s  %d waves/SIMD: %6.1f cycles per group\n",
           KIND < 2 ? (BIG ? "32x32x16" : "16x16x32") : "(no mfma)", NV, (KIND == 0 || KIND == 3) ? "v_exp_f32" : "v_fma_f32", w,
           cycles_per_group(ms, w, iters, 8));
}
template <int CH> void run_f64(int w)
{
    const int iters = 20000;
    const float ms = timed([](int g, int it) { hipLaunchKernelGGL((fma64<CH>), dim3(g), dim3(256), 0, 0, g_d, g_w, it); }, 256 * w, iters);
    printf("  v_fma_f64, %2d independent chains, %d waves/SIMD: %5.2f cycles per instruction\n", CH, w,
           cycles_per_group(ms, w, iters, 16));
}

// The same MFMA-only loop with operands that differ from one MFMA to the next (8 register pairs of pseudo-random
// bf16 values in [-2, 2)): what the chip sustains when the multipliers see data instead of constants.
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

// `issue_rates --mfma-peak`: one line, the bf16 matrix-core rate of this machine in TFLOP/s from the register-only
// loop of 32x32x16 MFMAs (8 independent accumulators, 2 wavefronts per SIMD), best of 5 launches.
static int mfma_peak()
{
    const int w = 2, iters = 20000;
    double best = 0.0;
    for (int rep = 0; rep < 5; ++rep) {
        const float ms = timed([](int g, int it) { hipLaunchKernelGGL((mfma_valu<0, 1, true>), dim3(g), dim3(256), 0, 0, g_f, it); },
                               256 * w, iters);
        // work-groups x wavefronts x iterations x 8 MFMAs x 2*32*32*16 FLOP
        const double flop = 256.0 * w * 4.0 * iters * 8.0 * 32768.0;
        best = flop / (ms * 1e-3) / 1e12 > best ? flop / (ms * 1e-3) / 1e12 : best;
    }
    // second figure: random operands, long enough (about 50 ms per launch) for the clock to settle
    double best_rand = 0.0;
    const int riters = 200000;
    for (int rep = 0; rep < 3; ++rep) {
        const float ms = timed([](int g, int it) { hipLaunchKernelGGL(mfma_random_operands, dim3(g), dim3(256), 0, 0, g_f, it); },
                               256 * w, riters);
        const double tf = 256.0 * w * 4.0 * riters * 8.0 * 32768.0 / (ms * 1e-3) / 1e12;
        best_rand = tf > best_rand ? tf : best_rand;
    }
    printf("%.1f %.1f\n", best, best_rand);
    return 0;
}

int main(int argc, char** argv)
{
    CHECK(hipMalloc(&g_f, 1024));
    if (argc > 1 && std::string(argv[1]) == "--mfma-peak") return mfma_peak();
    CHECK(hipMalloc(&g_d, 1024));
    CHECK(hipMalloc(&g_w, 64 * 16 * 8));
    CHECK(hipMemset(g_w, 0, 64 * 16 * 8));
    printf("1. matrix core + vector ALU on one SIMD (group = 1 MFMA + NV vector instructions)\n");
    for (int w : {1, 2, 4}) {
        run_mv<0, 1, true>(w);
        run_mv<2, 0, true>(w); run_mv<4, 0, true>(w); run_mv<4, 3, true>(w);
        run_mv<8, 1, true>(w); run_mv<8, 2, true>(w); run_mv<16, 1, true>(w); run_mv<16, 2, true>(w);
    }
    run_mv<0, 1, false>(2); run_mv<2, 1, false>(2); run_mv<4, 1, false>(2); run_mv<8, 1, false>(2);
    printf("2. fp64 vector FMA: one wavefront alone issues one every ~16 cycles, whatever the number of chains\n");
    for (int w : {1, 2, 4, 8}) { run_f64<2>(w); run_f64<16>(w); }
    {
        const int w = 8, iters = 20000;
        const float ms = timed([](int g, int it) { hipLaunchKernelGGL(mfma64, dim3(g), dim3(256), 0, 0, g_d, it); }, 256 * w, iters);
        printf("3. v_mfma_f64_16x16x4, %d waves/SIMD: %.1f cycles per MFMA = %.2f per 64-lane FMA equivalent\n", w,
               cycles_per_group(ms, w, iters, 4), cycles_per_group(ms, w, iters, 4) / 16);
    }
    return 0;
}
