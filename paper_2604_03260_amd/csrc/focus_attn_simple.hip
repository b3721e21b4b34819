// fp32 vector attention kernel (no matrix cores): the path for fp32 inputs and an
// independent on-device cross-check of the MFMA kernel for bf16 inputs.
//
// One work-group owns one query tile (<= L.BQ queries of one membership class) and
// handles it in passes of BQ_VECTOR rows.
// A row is shared by d/32 adjacent lanes, each holding 32 of the d components
// of q and of the output accumulator.  Keys and values are gathered 32 at a
// time through the class-ordered position array into LDS as fp32; the allowed
// set is App. D Eq. 3 with top-k sets and the softmax is exact (Sec. 1), kept
// online per 32-key step.
#include "focus_internal.h"
#include "focus_tileplan.h"

namespace focus {

namespace {

constexpr int SUB = 32;   // keys per inner step

template <typename T> __device__ inline float to_f32(T v);
template <> __device__ inline float to_f32<float>(float v) { return v; }
template <> __device__ inline float to_f32<uint16_t>(uint16_t v) { return __uint_as_float(((uint32_t)v) << 16); }

__device__ inline uint16_t f32_to_bf16_rne(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);   // NaN stays NaN
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}
template <typename T> __device__ inline T from_f32(float v);
template <> __device__ inline float from_f32<float>(float v) { return v; }
template <> __device__ inline uint16_t from_f32<uint16_t>(float v) { return f32_to_bf16_rne(v); }

template <typename T, int D>
__global__ __launch_bounds__(BQ_VECTOR * (D / 32)) void attn_simple_kernel(Layout L, HeadMap hm, const T* __restrict__ q,
                                                                    const T* __restrict__ k, const T* __restrict__ v,
                                                                    const char* __restrict__ ws, T* __restrict__ out,
                                                                    float* __restrict__ lse,
                                                                    int32_t* __restrict__ row_pairs)
{
    constexpr int TPR = D / 32;
    constexpr int NTHR = BQ_VECTOR * TPR;
    __shared__ TilePlan P;
    __shared__ __align__(16) float s_k[SUB * D];
    __shared__ __align__(16) float s_v[SUB * D];
    __shared__ int s_kpos[SUB];

    const int tid = threadIdx.x;
    const int job = blockIdx.x;
    const int bhq = blockIdx.y;
    const int b = bhq / L.Hq, h = bhq % L.Hq;
    const int bhk = b * L.Hkv + hm.kv[h];
    if (!plan_query_tile(L, ws, bhq, bhk, job, P)) return;

    for (int pass = 0; pass * BQ_VECTOR < P.nvalid; ++pass) {
    const int row = pass * BQ_VECTOR + tid / TPR, part = tid % TPR;
    const bool rvalid = row < P.nvalid;
    const int* qperm = (const int*)(ws + L.off_qperm) + (size_t)bhq * L.NQP;
    const int qpos = rvalid ? qperm[P.row0 + row] : -1;
    const int* kpos_all = (const int*)(ws + L.off_kpos) + (size_t)bhk * L.NKP;
    const T* kbase = k + (size_t)bhk * L.n * D;
    const T* vbase = v + (size_t)bhk * L.n * D;

    float qv[32], o[32];
#pragma unroll
    for (int e = 0; e < 32; ++e) {
        qv[e] = rvalid ? to_f32<T>(q[((size_t)bhq * L.n + qpos) * D + part * 32 + e]) : 0.f;
        o[e] = 0.f;
    }
    float m = -INFINITY, l = 0.f;
    int npairs = 0;
    const float scale = L.scale, cap = L.softcap;
    const int w = L.window;

    int cur = 0;
    for (int it = 0; it < P.total; ++it) {
        while (it >= P.cum[cur + 1]) ++cur;
        const int tile = P.t0[cur] + (it - P.cum[cur]);
        const bool inter = P.inter[cur] != 0;
        for (int sub = 0; sub < KT / SUB; ++sub) {
            const int r0 = tile * KT + sub * SUB;
            __syncthreads();
            if (tid < SUB) s_kpos[tid] = kpos_all[r0 + tid];
            for (int e = tid; e < SUB * D; e += NTHR) {
                const int kk = e / D, t = e % D;
                const int kp = kpos_all[r0 + kk];
                const bool real = kp != KPOS_PAD;
                s_k[e] = real ? to_f32<T>(kbase[(size_t)kp * D + t]) : 0.f;
                s_v[e] = real ? to_f32<T>(vbase[(size_t)kp * D + t]) : 0.f;
            }
            __syncthreads();
            float s[SUB];
            float mx = -INFINITY;
#pragma unroll
            for (int kk = 0; kk < SUB; ++kk) {
                float dot = 0.f;
                const float* kr = s_k + kk * D + part * 32;
#pragma unroll
                for (int e = 0; e < 32; ++e) dot = fmaf(qv[e], kr[e], dot);
#pragma unroll
                for (int off = 1; off < TPR; off <<= 1) dot += __shfl_xor(dot, off, 64);
                float x = dot * scale;
                if (cap > 0.f) x = cap * tanhf(x / cap);
                const int kp = s_kpos[kk];
                const bool ok = rvalid && kp <= qpos && (inter || kp > qpos - w);
                s[kk] = ok ? x : -INFINITY;
                npairs += ok ? 1 : 0;
                mx = fmaxf(mx, s[kk]);
            }
            const float m_new = fmaxf(m, mx);
            if (m_new == -INFINITY) continue;            // nothing allowed yet for this row
            const float alpha = expf(m - m_new);         // m = -inf gives 0
            float psum = 0.f;
#pragma unroll
            for (int kk = 0; kk < SUB; ++kk) {
                s[kk] = expf(s[kk] - m_new);             // masked: exp(-inf) = 0
                psum += s[kk];
            }
            l = l * alpha + psum;
            m = m_new;
#pragma unroll
            for (int e = 0; e < 32; ++e) o[e] *= alpha;
#pragma unroll
            for (int kk = 0; kk < SUB; ++kk) {
                const float* vr = s_v + kk * D + part * 32;
                const float pk = s[kk];
#pragma unroll
                for (int e = 0; e < 32; ++e) o[e] = fmaf(pk, vr[e], o[e]);
            }
        }
    }
    if (rvalid) {
    const float inv = 1.f / l;
    T* orow = out + ((size_t)bhq * L.n + qpos) * D + part * 32;
#pragma unroll
    for (int e = 0; e < 32; ++e) orow[e] = from_f32<T>(o[e] * inv);
    if (part == 0) {
        if (lse) lse[(size_t)bhq * L.n + qpos] = m + logf(l);
        if (row_pairs) row_pairs[(size_t)bhq * L.n + qpos] = npairs;
    }
    }
    }   // pass
}

}  // namespace

hipError_t launch_attn_simple(const Layout& L, const HeadMap& hm, const void* q, const void* k, const void* v,
                              char* ws, void* out, float* lse, int32_t* row_pairs, hipStream_t st)
{
    dim3 grid(L.NT, L.B * L.Hq);
#define FOCUS_LAUNCH_SIMPLE(T, D)                                                                      \
    hipLaunchKernelGGL((attn_simple_kernel<T, D>), grid, dim3(BQ_VECTOR*(D / 32)), 0, st, L, hm, (const T*)q, \
                       (const T*)k, (const T*)v, (const char*)ws, (T*)out, lse, row_pairs)
    if (L.dtype == 0) {
        if (L.d == 64) FOCUS_LAUNCH_SIMPLE(float, 64); else FOCUS_LAUNCH_SIMPLE(float, 128);
    } else {
        if (L.d == 64) FOCUS_LAUNCH_SIMPLE(uint16_t, 64); else FOCUS_LAUNCH_SIMPLE(uint16_t, 128);
    }
#undef FOCUS_LAUNCH_SIMPLE
    return hipGetLastError();
}

}  // namespace focus
