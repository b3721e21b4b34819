// fp32 vector attention kernel (no matrix cores): the path for fp32 inputs and an
// independent on-device cross-check of the MFMA kernel for bf16 inputs.
//
// One work-group owns one query tile (<= L.BQ queries of one membership class) and
// handles it in passes of BQ_VECTOR rows.
// A row is shared by D/32 adjacent lanes (D = head dim rounded up to 64, 128 or 256, zeros past d),
// each holding 32 of the components of q and of the output accumulator.  Keys and values are gathered
// SUB at a time through the class-ordered position array into LDS as fp32; the allowed
// set is App. D Eq. 3 with top-k sets and the softmax is exact (Sec. 1), kept
// online per 32-key step.
#include "focus_internal.h"
#include "focus_tileplan.h"

namespace focus {

namespace {

template <typename T> __device__ inline float to_f32(T v);
template <> __device__ inline float to_f32<float>(float v) { return v; }
template <> __device__ inline float to_f32<uint16_t>(uint16_t v) { return __uint_as_float(((uint32_t)v) << 16); }
template <> __device__ inline float to_f32<f16_bits>(f16_bits v) { return f16_bits_to_f32(v.v); }

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
template <> __device__ inline f16_bits from_f32<f16_bits>(float v) { return f16_bits{f32_to_f16_bits(v)}; }

// SUB: keys per inner step (the fp32 staging of a step's keys and values fills 2 * SUB * D * 4 bytes of LDS)
template <typename T, int D, int SUB>
__global__ __launch_bounds__(BQ_VECTOR * (D / 32)) void attn_simple_kernel(Layout L, HeadMap hm, const T* __restrict__ q,
                                                                    const T* __restrict__ k, const T* __restrict__ v,
                                                                    const float* __restrict__ g,
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
    const uint32_t mq_row = rvalid ? ((const uint32_t*)(ws + L.off_mq))[(size_t)bhq * L.n + qpos] : 0u;
    const uint32_t* mk_all = (const uint32_t*)(ws + L.off_mk) + (size_t)bhk * L.n;
    const int* kpos_all = (const int*)(ws + L.off_kpos) + (size_t)bhk * L.NKP;
    const int d = L.d;
    const size_t koff = (size_t)b * L.ks[0] + (size_t)hm.kv[h] * L.ks[1];
    const T* kbase = k + koff;
    const T* vbase = v + koff;
    const size_t kpitch = (size_t)L.ks[2];

    float qv[32], o[32];
#pragma unroll
    for (int e = 0; e < 32; ++e) {
        qv[e] = (rvalid && part * 32 + e < d)
                    ? to_f32<T>(q[(size_t)b * L.qs[0] + (size_t)h * L.qs[1] + (size_t)qpos * L.qs[2] + part * 32 + e]) : 0.f;
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
                const bool real = kp != KPOS_PAD && t < d;
                s_k[e] = real ? to_f32<T>(kbase[(size_t)kp * kpitch + t]) : 0.f;
                s_v[e] = real ? to_f32<T>(vbase[(size_t)kp * kpitch + t]) : 0.f;
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
                const int dlt = qpos - kp;               // pads sit at INT_MAX
                if (L.soft) {
                    // Sec. 2 Eq. 2: every causal pair; outside the window the score is scaled by
                    // sigmoid(lambda * g_i . g_j) = 1 / (1 + 2^(gate_slope * g_i . g_j))
                    const bool okc = rvalid && kp != KPOS_PAD && dlt >= 0;
                    if (okc && dlt >= w) {
                        const float* gi = g + ((size_t)b * L.n + qpos) * L.K;
                        const float* gj = g + ((size_t)b * L.n + kp) * L.K;
                        float aff = 0.f;
                        for (int c = 0; c < L.K; ++c) aff = fmaf(gi[c], gj[c], aff);
                        x *= 1.f / (1.f + exp2f(L.gate_slope * aff));
                    }
                    s[kk] = okc ? x : -INFINITY;
                    npairs += okc ? 1 : 0;
                    mx = fmaxf(mx, s[kk]);
                    continue;
                }
                bool share = inter;                      // exact classes: a common group is a class property
                if (L.coarse && inter && kp != KPOS_PAD) share = (mq_row & mk_all[kp]) != 0u;
                const bool loc = L.causal ? (dlt >= 0 && dlt < w) : (dlt < w && -dlt < w);
                const bool cz = L.causal ? dlt >= 0 : true;
                bool pair_ok = cz && (share || loc);
                // coarse classes that share a super-group hold pairs of both sets of a restricted launch
                if (L.coarse && inter && L.pair_set != 0) pair_ok = (L.pair_set == 1) ? (cz && share) : (loc && !share);
                const bool ok = rvalid && kp != KPOS_PAD && pair_ok;
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
    const float inv = (l > 0.f) ? 1.f / l : 0.f;     // empty row (launch restricted to one pair set): out = 0, lse = -inf
    T* orow = out + (size_t)b * L.os[0] + (size_t)h * L.os[1] + (size_t)qpos * L.os[2] + part * 32;
#pragma unroll
    for (int e = 0; e < 32; ++e)
        if (part * 32 + e < d) orow[e] = from_f32<T>(o[e] * inv);
    if (part == 0) {
        if (lse) lse[(size_t)bhq * L.n + qpos] = m + logf(l);
        if (row_pairs) row_pairs[(size_t)bhq * L.n + qpos] = npairs;
    }
    }
    }   // pass
}

// 8 consecutive components of a row (16-byte aligned: d is a multiple of 8) as fp32 and back
__device__ inline void load8(const float* p, float (&x)[8])
{
    const float4 a = *(const float4*)p, b = *(const float4*)(p + 4);
    x[0] = a.x; x[1] = a.y; x[2] = a.z; x[3] = a.w; x[4] = b.x; x[5] = b.y; x[6] = b.z; x[7] = b.w;
}
__device__ inline void load8(const uint16_t* p, float (&x)[8])
{
    const uint4 u = *(const uint4*)p;
    const uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        x[2 * e] = __uint_as_float(w[e] << 16);
        x[2 * e + 1] = __uint_as_float(w[e] & 0xffff0000u);
    }
}
__device__ inline void load8(const f16_bits* p, float (&x)[8])
{
    const uint4 u = *(const uint4*)p;
    const uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        x[2 * e] = f16_bits_to_f32((uint16_t)(w[e] & 0xffffu));
        x[2 * e + 1] = f16_bits_to_f32((uint16_t)(w[e] >> 16));
    }
}
__device__ inline void store8(f16_bits* p, const float (&y)[8])
{
    uint4 u;
    u.x = f32_to_f16_bits(y[0]) | ((uint32_t)f32_to_f16_bits(y[1]) << 16);
    u.y = f32_to_f16_bits(y[2]) | ((uint32_t)f32_to_f16_bits(y[3]) << 16);
    u.z = f32_to_f16_bits(y[4]) | ((uint32_t)f32_to_f16_bits(y[5]) << 16);
    u.w = f32_to_f16_bits(y[6]) | ((uint32_t)f32_to_f16_bits(y[7]) << 16);
    *(uint4*)p = u;
}
__device__ inline void store8(float* p, const float (&y)[8])
{
    *(float4*)p = make_float4(y[0], y[1], y[2], y[3]);
    *(float4*)(p + 4) = make_float4(y[4], y[5], y[6], y[7]);
}
__device__ inline void store8(uint16_t* p, const float (&y)[8])
{
    uint4 u;
    u.x = f32_to_bf16_rne(y[0]) | ((uint32_t)f32_to_bf16_rne(y[1]) << 16);
    u.y = f32_to_bf16_rne(y[2]) | ((uint32_t)f32_to_bf16_rne(y[3]) << 16);
    u.z = f32_to_bf16_rne(y[4]) | ((uint32_t)f32_to_bf16_rne(y[5]) << 16);
    u.w = f32_to_bf16_rne(y[6]) | ((uint32_t)f32_to_bf16_rne(y[7]) << 16);
    *(uint4*)p = u;
}

// App. D "Merge": two partial attentions over disjoint pair sets with their log-sum-exp values give
// the attention over the union, o = (e^{lA} oA + e^{lB} oB) / (e^{lA} + e^{lB}).  One thread per
// 8 consecutive components of a row; an empty part (lse = -inf) weighs nothing.
template <typename T>
__global__ __launch_bounds__(256) void attn_merge_kernel(size_t rows, int d, const T* __restrict__ oa,
                                                         const float* __restrict__ la, const T* __restrict__ ob,
                                                         const float* __restrict__ lb, T* __restrict__ out,
                                                         float* __restrict__ lse)
{
    const int cpr = d / 8;
    const size_t total = rows * (size_t)cpr;
    for (size_t id = (size_t)blockIdx.x * blockDim.x + threadIdx.x; id < total; id += (size_t)gridDim.x * blockDim.x) {
        const size_t r = id / cpr;
        const int c = (int)(id % cpr);
        const float a = la[r], b = lb[r];
        const float m = fmaxf(a, b);
        float wa = 0.f, wb = 0.f, l = -INFINITY;
        if (m != -INFINITY) {
            const float ea = expf(a - m), eb = expf(b - m);
            const float inv = 1.f / (ea + eb);
            wa = ea * inv;
            wb = eb * inv;
            l = m + logf(ea + eb);
        }
        const T* pa = oa + r * d + c * 8;
        const T* pb = ob + r * d + c * 8;
        T* po = out + r * d + c * 8;
        float xa[8], xb[8], y[8];
        load8(pa, xa);
        load8(pb, xb);
#pragma unroll
        for (int e = 0; e < 8; ++e) y[e] = wa * xa[e] + wb * xb[e];
        store8(po, y);
        if (c == 0 && lse) lse[r] = l;
    }
}

}  // namespace

hipError_t launch_attn_merge(size_t rows, int d, int dtype, const void* oa, const float* la, const void* ob,
                             const float* lb, void* out, float* lse, hipStream_t st)
{
    const size_t total = rows * (size_t)(d / 8);
    const unsigned grid = (unsigned)min((size_t)(256 * 64), (total + 255) / 256);
    if (dtype == 0)
        hipLaunchKernelGGL(attn_merge_kernel<float>, dim3(grid), dim3(256), 0, st, rows, d, (const float*)oa, la,
                           (const float*)ob, lb, (float*)out, lse);
    else if (dtype == 2)
        hipLaunchKernelGGL(attn_merge_kernel<f16_bits>, dim3(grid), dim3(256), 0, st, rows, d, (const f16_bits*)oa, la,
                           (const f16_bits*)ob, lb, (f16_bits*)out, lse);
    else
        hipLaunchKernelGGL(attn_merge_kernel<uint16_t>, dim3(grid), dim3(256), 0, st, rows, d, (const uint16_t*)oa, la,
                           (const uint16_t*)ob, lb, (uint16_t*)out, lse);
    return hipGetLastError();
}

hipError_t launch_attn_simple(const Layout& L, const HeadMap& hm, const void* q, const void* k, const void* v,
                              const float* g, char* ws, void* out, float* lse, int32_t* row_pairs, hipStream_t st)
{
    dim3 grid(L.NT, L.B * L.Hq);
#define FOCUS_LAUNCH_SIMPLE(T, D, SUB)                                                                 \
    hipLaunchKernelGGL((attn_simple_kernel<T, D, SUB>), grid, dim3(BQ_VECTOR*(D / 32)), 0, st, L, hm, (const T*)q, \
                       (const T*)k, (const T*)v, g, (const char*)ws, (T*)out, lse, row_pairs)
#define FOCUS_LAUNCH_SIMPLE_T(T)                                                                       \
    do {                                                                                               \
        if (L.dp == 64) FOCUS_LAUNCH_SIMPLE(T, 64, 32);                                                \
        else if (L.dp == 128) FOCUS_LAUNCH_SIMPLE(T, 128, 32);                                         \
        else FOCUS_LAUNCH_SIMPLE(T, 256, 16);                                                          \
    } while (0)
    if (L.dtype == 0) FOCUS_LAUNCH_SIMPLE_T(float);
    else if (L.dtype == 2) FOCUS_LAUNCH_SIMPLE_T(f16_bits);
    else FOCUS_LAUNCH_SIMPLE_T(uint16_t);
#undef FOCUS_LAUNCH_SIMPLE_T
#undef FOCUS_LAUNCH_SIMPLE
    return hipGetLastError();
}

}  // namespace focus
