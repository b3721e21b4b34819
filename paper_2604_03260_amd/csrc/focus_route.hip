// focus_route: the per-layer router (Sec. 2 Eq. 1 and the Sinkhorn recipe under it).
//
//   z_i = W_g^T h_i,  S[i,g] = z_i . C[g],  then either g_i = S[i,:] / tau (no normalisation)
//   or Q = exp(S / tau) followed by N rounds of {columns / their sum over the sequence's tokens,
//   rows / their sum over the groups}; the top-k entries of a row become the token's membership.
//
// Everything is fp64.  The projection is the plain inner product of Eq. 1: its products are exact
// (fp32 x bf16/fp16/fp32 fits in fp64) and are added one by one in index order t = 0 .. d_model-1 (one
// fused multiply-add per term, which rounds once, like an exact product followed by an add), so z, S
// and, without Sinkhorn, the membership are reproducible bit for bit.
//
// Kernels:
//   to_f64            W_g and C as fp64 tables (wave-uniform operands come from scalar loads);
//   route_project     one wavefront = 64 tokens (one per lane) x JW router outputs; hidden rows are
//                     streamed once through LDS in 64-component chunks (coalesced 16-byte loads, register
//                     prefetch of the next chunk, double-buffered LDS, one barrier per chunk); writes S,
//                     the work-group's largest score, and the masks directly when no Sinkhorn is asked;
//   route_max         largest score of each sequence (the shift that keeps exp finite; the first
//                     column step divides it out again);
//   sinkhorn_pass     Sinkhorn as diagonal scaling: Q = diag(u) E diag(v) with E = exp((S - max)/tau).
//                     A round is  v_g = 1 / sum_i u_i E[i,g],  u_i = 1 / sum_g E[i,g] v_g,  so one pass
//                     over E per round: every work-group first folds the previous pass's per-block
//                     column partial sums (fixed order, no atomics: deterministic), then updates its
//                     rows and leaves its own partial sums for the next pass.  The last pass writes
//                     the masks (ties to the smaller group index) and, if asked, the soft assignment.
#include "focus_internal.h"
#include <mutex>
#include <type_traits>

namespace focus {

// Scratch of focus_route_noalloc: device memory of the library's own image, one copy per GPU, held until the
// process ends.  Host code never uses this name as an address: route_static_scratch() asks the runtime for the
// array's device address once per device and hands that pointer to the kernels like any workspace.
static __device__ __align__(256) unsigned char scratch[ROUTE_STATIC_SCRATCH_BYTES];

hipError_t route_static_scratch(char** ptr)
{
    constexpr int MAX_DEVICES = 64;
    static std::mutex mu;
    static char* per_device[MAX_DEVICES] = {};
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= MAX_DEVICES) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(mu);
    if (!per_device[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));      // the copy of the array on the current device
        if (e != hipSuccess) return e;
        if (!p || ((uintptr_t)p & 255) != 0) return hipErrorInvalidSymbol;
        per_device[dev] = (char*)p;
    }
    *ptr = per_device[dev];
    return hipSuccess;
}

namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int RT = 64;                       // tokens per work-group of the projection (one per lane)
constexpr int RC = 64;                       // hidden components per LDS stage (staging only: the sum runs on across stages)

__global__ void to_f64_kernel(const float* __restrict__ src, double* __restrict__ dst, size_t count)
{
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t step = (size_t)gridDim.x * blockDim.x;
    for (; i < count; i += step) dst[i] = (double)src[i];
}

__device__ inline double wave_max(double x)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) x = fmax(x, __shfl_xor(x, off, 64));
    return x;
}

__device__ inline double wave_sum(double x)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) x = __dadd_rn(x, __shfl_xor(x, off, 64));
    return x;
}

// top-k of the first K of KP register values by rank counting; ties go to the smaller index
template <int KP>
__device__ inline uint32_t topk_mask(const double (&s)[KP], int K, int topk)
{
    uint32_t m = 0;
#pragma unroll
    for (int g = 0; g < KP; ++g) {
        int beaten = 0;
#pragma unroll
        for (int o = 0; o < KP; ++o)
            if (o != g) beaten += (o < K && (s[o] > s[g] || (s[o] == s[g] && o < g))) ? 1 : 0;
        if (g < K && beaten < topk) m |= (1u << g);
    }
    if (__popc(m) != topk) m = (topk == 32) ? 0xffffffffu : ((1u << topk) - 1u);   // a NaN among the scores
    return m;
}

// ---------------------------------------------------------------- projection + scores
template <typename T, int JW, int NW>
__global__ __launch_bounds__(64 * NW) void route_project_kernel(RouteLayout R, const T* __restrict__ hidden,
                                                                 const double* __restrict__ w64,
                                                                 const double* __restrict__ c64,
                                                                 char* __restrict__ ws,
                                                                 uint32_t* __restrict__ masks,
                                                                 double* __restrict__ soft)
{
    constexpr int DG = JW * NW;
    constexpr int NTHR = 64 * NW;
    constexpr int ROW_BYTES = RC * (int)sizeof(T);
    constexpr int ROW_STRIDE = ROW_BYTES + 16;
    constexpr int CPR = ROW_BYTES / 16;                  // 16-byte pieces per staged row
    constexpr int LPT = RT * CPR / NTHR;                 // pieces per thread
    constexpr int EPC = 16 / (int)sizeof(T);
    // dynamic LDS: two staging buffers during the projection, then z [RT][DG+1] and S [RT][K|1] in their place
    extern __shared__ __align__(16) char s_dyn[];
    __shared__ double s_wmax[NW];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int b = blockIdx.y;
    const int tok0 = blockIdx.x * RT;
    const int n = R.n, dm = R.dm, K = R.K;
    const int rows = min(RT, n - tok0);
    const int row_bytes = dm * (int)sizeof(T);
    const char* gbase = (const char*)hidden + ((size_t)b * n + tok0) * row_bytes;
    const int nchunk = (dm + RC - 1) / RC;

    u32x4 st[LPT];
#define FOCUS_ROUTE_LOAD(CH)                                                                          \
    do {                                                                                              \
        _Pragma("unroll") for (int i = 0; i < LPT; ++i) {                                             \
            const int pid_ = tid + i * NTHR;                                                          \
            const int r_ = pid_ / CPR, cc_ = pid_ % CPR;                                              \
            const int byte_ = (CH) * ROW_BYTES + cc_ * 16;                                            \
            const u32x4 z_ = {0u, 0u, 0u, 0u};                                                        \
            st[i] = (r_ < rows && byte_ < row_bytes) ? *(const u32x4*)(gbase + (size_t)r_ * row_bytes + byte_) : z_; \
        }                                                                                             \
    } while (0)

    double acc[JW];
#pragma unroll
    for (int j = 0; j < JW; ++j) acc[j] = 0.0;

    FOCUS_ROUTE_LOAD(0);
    for (int ch = 0; ch < nchunk; ++ch) {
        char* buf = s_dyn + (ch & 1) * (RT * ROW_STRIDE);
#pragma unroll
        for (int i = 0; i < LPT; ++i) {
            const int pid = tid + i * NTHR;
            *(u32x4*)(buf + (pid / CPR) * ROW_STRIDE + (pid % CPR) * 16) = st[i];
        }
        __syncthreads();               // also orders this write after every wave's reads two chunks ago
        if (ch + 1 < nchunk) FOCUS_ROUTE_LOAD(ch + 1);
        const int tbase = ch * RC;
        const int tcount = min(RC, dm - tbase);          // dm is a multiple of 8: whole pieces only
#pragma unroll 1
        for (int cc = 0; cc * EPC < tcount; ++cc) {
            const u32x4 val = *(const u32x4*)(buf + lane * ROW_STRIDE + cc * 16);
            double xv[EPC];
            if constexpr (sizeof(T) == 4) {
#pragma unroll
                for (int e = 0; e < 4; ++e) xv[e] = (double)__uint_as_float(val[e]);
            } else if constexpr (std::is_same<T, f16_bits>::value) {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    xv[2 * e] = (double)f16_bits_to_f32((uint16_t)(val[e] & 0xffffu));
                    xv[2 * e + 1] = (double)f16_bits_to_f32((uint16_t)(val[e] >> 16));
                }
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    xv[2 * e] = (double)__uint_as_float(val[e] << 16);
                    xv[2 * e + 1] = (double)__uint_as_float(val[e] & 0xffff0000u);
                }
            }
#pragma unroll
            for (int e = 0; e < EPC; ++e) {
                const double* wr = w64 + (size_t)(tbase + cc * EPC + e) * DG + wave * JW;   // wave-uniform
#pragma unroll
                for (int j = 0; j < JW; ++j) acc[j] = fma(xv[e], wr[j], acc[j]);
            }
        }
    }
#undef FOCUS_ROUTE_LOAD

    // z of the 64 tokens -> LDS, then S[i,g] = sum_j z_j C[g][j] in index order (products rounded, then added)
    __syncthreads();                                     // the staging buffers are free
    double* s_z = (double*)s_dyn;
    double* s_s = s_z + RT * (DG + 1);
    const int KS = K | 1;
#pragma unroll
    for (int j = 0; j < JW; ++j) s_z[lane * (DG + 1) + wave * JW + j] = acc[j];
    __syncthreads();
    double mymax = -INFINITY;
    for (int g = wave; g < K; g += NW) {
        const double* cr = c64 + (size_t)g * DG;                                            // wave-uniform
        double s = 0.0;
#pragma unroll 4
        for (int j = 0; j < DG; ++j) s = __dadd_rn(s, __dmul_rn(s_z[lane * (DG + 1) + j], cr[j]));
        s_s[lane * KS + g] = s;
        if (lane < rows) mymax = fmax(mymax, s);
    }
    mymax = wave_max(mymax);
    if (lane == 0) s_wmax[wave] = mymax;
    __syncthreads();
    if (tid == 0) {
        double m = s_wmax[0];
        for (int w = 1; w < NW; ++w) m = fmax(m, s_wmax[w]);
        ((double*)(ws + R.off_maxpart))[(size_t)b * R.nproj + blockIdx.x] = m;
    }
    if (tid < rows) {
        const size_t tok = (size_t)b * n + tok0 + tid;
        double* mine = s_s + tid * KS;
        if (R.iters == 0) {
            for (int g = 0; g < K; ++g) mine[g] = mine[g] / R.tau;
            uint32_t m = 0;
            for (int g = 0; g < K; ++g) {
                const double sg = mine[g];
                int beaten = 0;
                for (int o = 0; o < K; ++o) {
                    const double so = mine[o];
                    beaten += (o != g && (so > sg || (so == sg && o < g))) ? 1 : 0;
                }
                if (beaten < R.topk) m |= (1u << g);
            }
            if (__popc(m) != R.topk) m = (R.topk == 32) ? 0xffffffffu : ((1u << R.topk) - 1u);   // NaN scores
            masks[tok] = m;
            if (soft) for (int g = 0; g < K; ++g) soft[tok * K + g] = mine[g];
        } else {
            double* Srow = (double*)(ws + R.off_S) + tok * K;
            for (int g = 0; g < K; ++g) Srow[g] = mine[g];
        }
    }
}

// largest score of each sequence
__global__ __launch_bounds__(256) void route_max_kernel(RouteLayout R, char* __restrict__ ws)
{
    __shared__ double s_w[4];
    const int tid = threadIdx.x, b = blockIdx.x;
    const double* mp = (const double*)(ws + R.off_maxpart) + (size_t)b * R.nproj;
    double m = -INFINITY;
    for (int i = tid; i < R.nproj; i += 256) m = fmax(m, mp[i]);
    m = wave_max(m);
    if ((tid & 63) == 0) s_w[tid >> 6] = m;
    __syncthreads();
    if (tid == 0) ((double*)(ws + R.off_smax))[b] = fmax(fmax(s_w[0], s_w[1]), fmax(s_w[2], s_w[3]));
}

// ---------------------------------------------------------------- Sinkhorn passes
// pass 0: E = exp((S - max)/tau) in place, column partial sums of E.
// pass t = 1..N: v from the partial sums of pass t-1, u per row, partial sums of u E (or, on pass N, the outputs).
template <int KP>
__global__ __launch_bounds__(256) void sinkhorn_pass_kernel(RouteLayout R, int pass, char* __restrict__ ws,
                                                            uint32_t* __restrict__ masks, double* __restrict__ soft)
{
    __shared__ double s_v[KP];
    __shared__ double s_part[4][KP];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int blk = blockIdx.x, b = blockIdx.y;
    const int n = R.n, K = R.K;
    double* E = (double*)(ws + R.off_S) + (size_t)b * n * K;
    const double* prev = (const double*)(ws + R.off_colpart) + ((size_t)((pass + 1) & 1) * R.B + b) * R.nsink * KP;
    double* mine = (double*)(ws + R.off_colpart) + (((size_t)(pass & 1) * R.B + b) * R.nsink + blk) * KP;
    const bool last = pass == R.iters;

    if (pass > 0) {
        for (int g = wave; g < K; g += 4) {
            double s = 0.0;
            for (int i = lane; i < R.nsink; i += 64) s = __dadd_rn(s, prev[(size_t)i * KP + g]);
            s = wave_sum(s);
            if (lane == 0) s_v[g] = 1.0 / s;
        }
        __syncthreads();
    }
    const double smax = ((const double*)(ws + R.off_smax))[b];
    double v[KP], cs[KP];
#pragma unroll
    for (int g = 0; g < KP; ++g) {
        v[g] = (pass > 0 && g < K) ? s_v[g] : 1.0;
        cs[g] = 0.0;
    }
    const int t_end = min(n, (blk + 1) * R.sink_tokens);
    for (int i = blk * R.sink_tokens + tid; i < t_end; i += 256) {
        double e[KP];
        double* row = E + (size_t)i * K;
        if (pass == 0) {
#pragma unroll
            for (int g = 0; g < KP; ++g)
                if (g < K) {
                    e[g] = exp((row[g] - smax) / R.tau);
                    row[g] = e[g];
                    cs[g] = __dadd_rn(cs[g], e[g]);
                }
            continue;
        }
        double rs = 0.0;
#pragma unroll
        for (int g = 0; g < KP; ++g) {
            e[g] = (g < K) ? __dmul_rn(row[g], v[g]) : 0.0;
            rs = __dadd_rn(rs, e[g]);
        }
        const double u = 1.0 / rs;
        if (!last) {
#pragma unroll
            for (int g = 0; g < KP; ++g)
                if (g < K) cs[g] = __dadd_rn(cs[g], __dmul_rn(u, row[g]));
        } else {
            const size_t tok = (size_t)b * n + i;
#pragma unroll
            for (int g = 0; g < KP; ++g) e[g] = __dmul_rn(e[g], u);
            masks[tok] = topk_mask<KP>(e, K, R.topk);
            if (soft) {
#pragma unroll
                for (int g = 0; g < KP; ++g)
                    if (g < K) soft[tok * K + g] = e[g];
            }
        }
    }
    if (last && pass > 0) return;
#pragma unroll
    for (int g = 0; g < KP; ++g) {
        const double s = wave_sum(cs[g]);
        if (lane == 0) s_part[wave][g] = s;
    }
    __syncthreads();
    if (tid < K) mine[tid] = __dadd_rn(__dadd_rn(s_part[0][tid], s_part[1][tid]), __dadd_rn(s_part[2][tid], s_part[3][tid]));
}

template <typename T>
hipError_t launch_project(const RouteLayout& R, const void* hidden, char* ws, uint32_t* masks, double* soft,
                          hipStream_t st)
{
    const double* w64 = (const double*)(ws + R.off_w64);
    const double* c64 = (const double*)(ws + R.off_c64);
    dim3 grid(R.nproj, R.B);
    const size_t stage = 2 * (size_t)RT * (RC * sizeof(T) + 16);
    const size_t tail = (size_t)RT * (R.dg + 1 + (R.K | 1)) * sizeof(double);
    const size_t lds = stage > tail ? stage : tail;
#define FOCUS_PROJ(JW, NW)                                                                                   \
    hipLaunchKernelGGL((route_project_kernel<T, JW, NW>), grid, dim3(64 * NW), lds, st, R, (const T*)hidden, w64, \
                       c64, ws, masks, soft)
    // JW router outputs per wavefront: more of them amortise the fp64 conversion of every hidden value,
    // fewer give more wavefronts.  A wavefront issues one fp64 instruction about every 16 cycles, a SIMD
    // one every 4: the fp64 rate needs 4 or more wavefronts per SIMD, so the split follows the token count
    // (measured at d_model 4096..8192, d_g 16: 8 x 2 wins from 2048 groups of 64 tokens on, 4 x 4 below,
    // 16 x 1 nowhere).
    const long groups = (long)R.nproj * R.B;
    switch (R.dg) {
        case 4: FOCUS_PROJ(4, 1); break;
        case 8: FOCUS_PROJ(4, 2); break;
        case 16: if (groups >= 2048) FOCUS_PROJ(8, 2); else FOCUS_PROJ(4, 4); break;
        case 32: FOCUS_PROJ(8, 4); break;
        default: FOCUS_PROJ(16, 4); break;
    }
#undef FOCUS_PROJ
    return hipGetLastError();
}

}  // namespace

hipError_t launch_route(const RouteLayout& R, const void* hidden, const float* wg, const float* cent, char* ws,
                        uint32_t* masks, double* soft, hipStream_t st)
{
    hipError_t e;
    const size_t nw = (size_t)R.dm * R.dg, nc = (size_t)R.K * R.dg;
    hipLaunchKernelGGL(to_f64_kernel, dim3((unsigned)min((size_t)1024, (nw + 255) / 256)), dim3(256), 0, st, wg,
                       (double*)(ws + R.off_w64), nw);
    hipLaunchKernelGGL(to_f64_kernel, dim3(1), dim3(256), 0, st, cent, (double*)(ws + R.off_c64), nc);
    if (R.dtype == 0) e = launch_project<float>(R, hidden, ws, masks, soft, st);
    else if (R.dtype == 2) e = launch_project<f16_bits>(R, hidden, ws, masks, soft, st);
    else e = launch_project<uint16_t>(R, hidden, ws, masks, soft, st);
    if (e != hipSuccess) return e;
    if (R.iters == 0) return hipSuccess;
    hipLaunchKernelGGL(route_max_kernel, dim3(R.B), dim3(256), 0, st, R, ws);
    dim3 grid(R.nsink, R.B);
    for (int pass = 0; pass <= R.iters; ++pass) {
        if (R.K <= 4) hipLaunchKernelGGL((sinkhorn_pass_kernel<4>), grid, dim3(256), 0, st, R, pass, ws, masks, soft);
        else if (R.K <= 8) hipLaunchKernelGGL((sinkhorn_pass_kernel<8>), grid, dim3(256), 0, st, R, pass, ws, masks, soft);
        else if (R.K <= 16) hipLaunchKernelGGL((sinkhorn_pass_kernel<16>), grid, dim3(256), 0, st, R, pass, ws, masks, soft);
        else hipLaunchKernelGGL((sinkhorn_pass_kernel<32>), grid, dim3(256), 0, st, R, pass, ws, masks, soft);
    }
    return hipGetLastError();
}

}  // namespace focus
