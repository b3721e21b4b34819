// focus_decode: one new token per sequence against a key/value cache (incremental inference).
//
// The mask row of the newest token i (App. D Eq. 3 with top-k sets, the same predicate as the
// prefill path) is  { j <= i : i - j < w  or  Gq(i) and Gk(j) intersect }.  Memory-bound: every
// attended key costs its K row and its V row once.  The cache state keeps, per (batch, KV head),
// the membership mask of every cached key and one position list per group (positions are appended
// in order, so the lists stay ascending).  A step
//   1. routes the new key and the new queries (fp64 scores, summed in index order like the prefill
//      scoring, top-k with ties to the smaller group), writes the key's mask, appends its position
//      to the lists of its groups and copies the K and V rows into the caches;
//   2. attends: the keys of the window come straight from the caches; the keys before the window
//      come from the lists of the query's groups, cut at the window's lower edge (a per-list pointer that
//      step 1 advances with the window);
//      a key that sits in several of the query's groups is taken from the first of them only (its
//      mask tells).  The concatenation [window | list prefix of group 1 | group 2 | ...] is cut into
//      chunks of DEC_CHUNK keys with an online softmax per chunk.  When the lists together hold at least
//      as many entries as there are positions below the window (few groups, several of them per query),
//      the positions 0..pos are walked instead and every key's mask is tested against the query's;
//      grouped-query heads share one walk over the union of their keys, and 16-bit caches run both
//      products on the matrix cores;
//   3. merges the chunks' partial (o, max, sum) by their log-sum-exp weights (App. D "Merge", n-ary).
#include "focus_internal.h"
#include <algorithm>
#include <type_traits>

namespace focus {

namespace {

template <typename T> __device__ inline float dec_to_f32(T v);
template <> __device__ inline float dec_to_f32<float>(float v) { return v; }
template <> __device__ inline float dec_to_f32<uint16_t>(uint16_t v) { return __uint_as_float(((uint32_t)v) << 16); }
template <> __device__ inline float dec_to_f32<f16_bits>(f16_bits v) { return f16_bits_to_f32(v.v); }

__device__ inline uint16_t dec_bf16_rne(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}
template <typename T> __device__ inline T dec_from_f32(float v);
template <> __device__ inline float dec_from_f32<float>(float v) { return v; }
template <> __device__ inline uint16_t dec_from_f32<uint16_t>(float v) { return dec_bf16_rne(v); }
template <> __device__ inline f16_bits dec_from_f32<f16_bits>(float v) { return f16_bits{f32_to_f16_bits(v)}; }

// 8 consecutive components as fp32
__device__ inline void dec_load8(const float* p, float (&x)[8])
{
    const float4 a = *(const float4*)p, b = *(const float4*)(p + 4);
    x[0] = a.x; x[1] = a.y; x[2] = a.z; x[3] = a.w; x[4] = b.x; x[5] = b.y; x[6] = b.z; x[7] = b.w;
}
__device__ inline void dec_load8(const uint16_t* p, float (&x)[8])
{
    const uint4 u = *(const uint4*)p;
    const uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        x[2 * e] = __uint_as_float(w[e] << 16);
        x[2 * e + 1] = __uint_as_float(w[e] & 0xffff0000u);
    }
}

__device__ inline void dec_load8(const f16_bits* p, float (&x)[8])
{
    const uint4 u = *(const uint4*)p;
    const uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        x[2 * e] = f16_bits_to_f32((uint16_t)(w[e] & 0xffffu));
        x[2 * e + 1] = f16_bits_to_f32((uint16_t)(w[e] >> 16));
    }
}

// top-k mask of the scores held by lanes 0..K-1 of a wavefront (ties to the smaller group index)
__device__ inline uint32_t wave_topk_mask(double s, int lane, int K, int topk)
{
    int beaten = 0;
    for (int o = 0; o < K; ++o) {
        const double so = __shfl(s, o, 64);
        beaten += (o != lane && (so > s || (so == s && o < lane))) ? 1 : 0;
    }
    uint32_t member = (uint32_t)__ballot(lane < K && beaten < topk);
    // a NaN score loses no comparison: more than topk bits, replaced by the first topk groups
    if (__popc(member) != topk) member = (topk == 32) ? 0xffffffffu : ((1u << topk) - 1u);
    return member;
}

// A membership given from outside (the per-layer router) must be a topk-subset of the K groups: anything else
// would break the "every key sits in exactly topk lists" bound of the step; it is replaced by the first topk groups.
__device__ inline uint32_t decode_valid_mask(uint32_t m, int K, int topk)
{
    const uint32_t allowed = (K == 32) ? 0xffffffffu : ((1u << K) - 1u);
    if ((m & ~allowed) != 0u || __popc(m) != topk) m = (topk == 32) ? 0xffffffffu : ((1u << topk) - 1u);
    return m;
}

// membership of the cached keys from per-token masks [B, n_ctx]: every KV head of a token takes the token's mask
__global__ __launch_bounds__(256) void decode_prefill_masks_kernel(DecodeLayout L, int n_ctx,
                                                                   const uint32_t* __restrict__ token_masks,
                                                                   char* __restrict__ st)
{
    const int j = blockIdx.x * 256 + threadIdx.x;
    const int bhk = blockIdx.y, b = bhk / L.Hkv;
    if (j >= n_ctx) return;
    ((uint32_t*)(st + L.off_mk))[(size_t)bhk * L.n + j] = decode_valid_mask(token_masks[(size_t)b * n_ctx + j], L.K, L.topk);
}

__global__ void decode_zero_kernel(int* __restrict__ p, int count)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) p[i] = 0;
}

// ---------------------------------------------------------------- prefill of the cache state
// membership of the cached keys 0 .. n_ctx-1: one thread per key, fp64 scores in index order;
// KMAX = K rounded up, so that the scores stay in registers
template <typename T, int KMAX>
__global__ __launch_bounds__(256) void decode_prefill_score_kernel(DecodeLayout L, int n_ctx, const T* __restrict__ kc,
                                                                   const float* __restrict__ cents, char* __restrict__ st)
{
    const int j = blockIdx.x * 256 + threadIdx.x;
    const int bhk = blockIdx.y, hk = bhk % L.Hkv;
    if (j >= n_ctx) return;
    const int K = L.K;
    const T* row = kc + ((size_t)bhk * L.n + j) * L.d;
    const float* c = cents + (size_t)hk * K * L.d;        // wave-uniform: scalar loads
    double s[KMAX];
#pragma unroll
    for (int g = 0; g < KMAX; ++g) s[g] = 0.0;
    for (int t0 = 0; t0 < L.d; t0 += 8) {            // 16-byte (bf16) or 32-byte (fp32) pieces of the row, index order kept
        float xv[8];
        dec_load8(row + t0, xv);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const double x = (double)xv[e];
#pragma unroll
            for (int g = 0; g < KMAX; ++g)
                if (g < K) s[g] = fma(x, (double)c[(size_t)g * L.d + t0 + e], s[g]);
        }
    }
    uint32_t m = 0;
#pragma unroll
    for (int g = 0; g < KMAX; ++g) {
        int beaten = 0;
#pragma unroll
        for (int o = 0; o < KMAX; ++o) beaten += (o < K && o != g && (s[o] > s[g] || (s[o] == s[g] && o < g))) ? 1 : 0;
        if (g < K && beaten < L.topk) m |= (1u << g);
    }
    if (__popc(m) != L.topk) m = (L.topk == 32) ? 0xffffffffu : ((1u << L.topk) - 1u);   // NaN scores
    ((uint32_t*)(st + L.off_mk))[(size_t)bhk * L.n + j] = m;
}

// position list of one group of one (batch, KV head): ordered compaction, 256 positions per round
__global__ __launch_bounds__(256) void decode_prefill_lists_kernel(DecodeLayout L, int n_ctx, char* __restrict__ st)
{
    __shared__ int s_w[4];
    __shared__ int s_base;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int g = blockIdx.x, bhk = blockIdx.y;
    const uint32_t* mk = (const uint32_t*)(st + L.off_mk) + (size_t)bhk * L.n;
    int* list = (int*)(st + L.off_lists) + ((size_t)bhk * L.K + g) * L.n;
    if (tid == 0) s_base = 0;
    __syncthreads();
    // entries below the window of the next step (position n_ctx): positions < n_ctx - window + 1
    const int lo_next = n_ctx - L.window + 1;
    int below = 0;
    for (int j0 = 0; j0 < n_ctx; j0 += 256) {
        const int j = j0 + tid;
        const bool mine = j < n_ctx && ((mk[j] >> g) & 1u);
        below += (mine && j < lo_next) ? 1 : 0;
        const unsigned long long bal = __ballot(mine);
        const unsigned long long lt = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
        if (lane == 0) s_w[wave] = __popcll(bal);
        __syncthreads();
        int before = s_base;
        for (int w2 = 0; w2 < wave; ++w2) before += s_w[w2];
        if (mine) list[before + __popcll(bal & lt)] = j;
        __syncthreads();
        if (tid == 0) s_base += s_w[0] + s_w[1] + s_w[2] + s_w[3];
        __syncthreads();
    }
    if (tid == 0) ((int*)(st + L.off_counts))[(size_t)bhk * L.K + g] = s_base;
    // block-wide sum of `below` -> the group's window pointer
    __syncthreads();
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) below += __shfl_xor(below, off, 64);
    if (lane == 0) s_w[wave] = below;
    __syncthreads();
    if (tid == 0) ((int*)(st + L.off_wp))[(size_t)bhk * L.K + g] = s_w[0] + s_w[1] + s_w[2] + s_w[3];
}

// ---------------------------------------------------------------- step 1: route and append
// One wavefront per (batch, head): heads [0, Hq) are the new queries, [Hq, Hq + Hkv) the new keys.
// The vector and the K centroid rows are staged in LDS first, so the fp64 chain of lane g (group g,
// components in index order) runs from LDS instead of waiting for a global load per component.
template <typename T>
__global__ __launch_bounds__(64) void decode_route_kernel(DecodeLayout L, HeadMap hm, int pos_arg, const int* __restrict__ pos_dev,
                                                          const T* __restrict__ q_new,
                                                          const T* __restrict__ k_new, const T* __restrict__ v_new,
                                                          const float* __restrict__ cents,
                                                          const uint32_t* __restrict__ token_mask, T* __restrict__ kc,
                                                          T* __restrict__ vc, char* __restrict__ st)
{
    __shared__ float s_x[256];
    __shared__ float s_c[32 * 257];               // row stride d + 1: the K lanes read K different rows
    const int lane = threadIdx.x;
    // the position comes from the launch (one for all sequences), or from device memory, one per sequence,
    // when a captured graph serves every step or the sequences of a batch stand at different positions;
    // a position outside the caches makes the step skip that sequence (the host could not check it)
    const int b = blockIdx.y, hh = blockIdx.x;
    const int pos = pos_dev ? pos_dev[b] : pos_arg;
    if (pos < 0 || pos >= L.n) return;
    const bool is_q = hh < L.Hq;
    const int h = is_q ? hh : hh - L.Hq;
    const int hk = is_q ? hm.kv[h] : h;
    const int d = L.d;
    const T* x = is_q ? q_new + ((size_t)b * L.Hq + h) * d : k_new + ((size_t)b * L.Hkv + h) * d;
    const size_t bhk = (size_t)b * L.Hkv + h;     // KV-head wavefronts only
    // Everything that does not depend on the scores is loaded first, so that the scoring hides those round
    // trips: the vector itself, for a key also its V row, the lengths and window pointers of the lists and the
    // two list entries the window's lower edge can pass in this step.
    T xr[4], vr[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int t = lane + 64 * i;
        if (t < d) xr[i] = x[t];
        if (!is_q && t < d) vr[i] = v_new[bhk * d + t];
    }
    int cn = 0, w = 0, l0 = 0, l1 = 0;
    const int* list = (const int*)(st + L.off_lists) + (bhk * L.K + lane) * L.n;   // of group `lane`
    if (!is_q && lane < L.K) {
        cn = ((const int*)(st + L.off_counts))[bhk * L.K + lane];
        w = ((const int*)(st + L.off_wp))[bhk * L.K + lane];
        if (w < cn) l0 = list[w];
        if (w + 1 < cn) l1 = list[w + 1];
    }
    uint32_t mask;
    if (token_mask) {
        // the new token's membership comes from the per-layer router: the same for every head, as query and as key
        mask = decode_valid_mask(token_mask[b], L.K, L.topk);
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i)
            if (lane + 64 * i < d) s_x[lane + 64 * i] = dec_to_f32<T>(xr[i]);
        const float* c = cents + (size_t)hk * L.K * d;
        // eight loads in flight per lane (one at a time, the staging alone is a chain of K * d / 64 round trips)
        for (int e0 = lane; e0 < L.K * d; e0 += 64 * 8) {
            float cv[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) cv[i] = (e0 + 64 * i < L.K * d) ? c[e0 + 64 * i] : 0.f;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int e = e0 + 64 * i;
                if (e < L.K * d) s_c[(e / d) * (d + 1) + e % d] = cv[i];
            }
        }
        __syncthreads();
        double s = 0.0;
        if (lane < L.K) {
            // index order, eight components per LDS round trip (d is a multiple of 8)
            const float* cr = s_c + lane * (d + 1);
            for (int t = 0; t < d; t += 8) {
                float xs[8], cs[8];
#pragma unroll
                for (int i = 0; i < 8; ++i) { xs[i] = s_x[t + i]; cs[i] = cr[t + i]; }
#pragma unroll
                for (int i = 0; i < 8; ++i) s = fma((double)xs[i], (double)cs[i], s);
            }
        }
        mask = wave_topk_mask(s, lane, L.K, L.topk);
    }
    if (is_q) {
        if (lane == 0) ((uint32_t*)(st + L.off_mq))[(size_t)b * L.Hq + h] = mask;
        return;
    }
    if (lane == 0) ((uint32_t*)(st + L.off_mk))[bhk * L.n + pos] = mask;
    if (lane < L.K) {
        if ((mask >> lane) & 1u) {
            // single writer: this lane owns the group's list
            ((int*)(st + L.off_lists))[(bhk * L.K + lane) * L.n + cn] = pos;
            ((int*)(st + L.off_counts))[bhk * L.K + lane] = cn + 1;
        }
        // window pointer: number of list entries below this step's window, among the cn entries before this
        // step's append (pos itself is in the window).  The window's lower edge moves with pos and positions are
        // unique, so the pointer normally advances by at most one per step.
        const int lo_w = pos - L.window + 1;
        if (w < cn && l0 < lo_w) {
            ++w;
            if (w < cn && l1 < lo_w) {
                ++w;
                while (w < cn && list[w] < lo_w) ++w;
            }
        }
        ((int*)(st + L.off_wp))[bhk * L.K + lane] = w;
    }
    T* kdst = kc + (bhk * L.n + pos) * d;
    T* vdst = vc + (bhk * L.n + pos) * d;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int t = lane + 64 * i;
        if (t < d) { kdst[t] = xr[i]; vdst[t] = vr[i]; }
    }
}

// ---------------------------------------------------------------- step 2: attention over one chunk of the key sequence
// 8 consecutive components of a cache row, kept packed until they are used
template <typename T> struct Raw8;
template <> struct Raw8<uint16_t> {
    uint4 u;
    __device__ inline void load(const uint16_t* p) { u = *(const uint4*)p; }
    __device__ inline void zero() { u = make_uint4(0u, 0u, 0u, 0u); }
    __device__ inline void unpack(float (&x)[8]) const
    {
        const uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            x[2 * e] = __uint_as_float(w[e] << 16);
            x[2 * e + 1] = __uint_as_float(w[e] & 0xffff0000u);
        }
    }
};
template <> struct Raw8<f16_bits> {
    uint4 u;
    __device__ inline void load(const f16_bits* p) { u = *(const uint4*)p; }
    __device__ inline void zero() { u = make_uint4(0u, 0u, 0u, 0u); }
    __device__ inline void unpack(float (&x)[8]) const
    {
        const uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            x[2 * e] = f16_bits_to_f32((uint16_t)(w[e] & 0xffffu));
            x[2 * e + 1] = f16_bits_to_f32((uint16_t)(w[e] >> 16));
        }
    }
};
template <> struct Raw8<float> {
    float4 a, b;
    __device__ inline void load(const float* p) { a = *(const float4*)p; b = *(const float4*)(p + 4); }
    __device__ inline void zero() { a = make_float4(0.f, 0.f, 0.f, 0.f); b = a; }
    __device__ inline void unpack(float (&x)[8]) const
    {
        x[0] = a.x; x[1] = a.y; x[2] = a.z; x[3] = a.w; x[4] = b.x; x[5] = b.y; x[6] = b.z; x[7] = b.w;
    }
};

// lanes that share one key: a power of two covering d / 8 slices of 8 components (the lanes past d / 8 hold zeros)
__host__ __device__ constexpr int lanes_per_key(int d) { return d <= 64 ? 8 : d <= 128 ? 16 : 32; }

// sum over the LPK (8, 16 or 32) adjacent lanes that share a key, by DPP lane permutations (no LDS):
// xor 1, xor 2 inside quads, then mirror inside 8 lanes, then mirror inside the 16-lane row; two rows
// meet through a lane exchange
template <int LPK>
__device__ inline float slice_sum(float x)
{
    x += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0xB1, 0xF, 0xF, false));    // quad_perm [1,0,3,2]
    x += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x4E, 0xF, 0xF, false));    // quad_perm [2,3,0,1]
    x += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x141, 0xF, 0xF, false));   // row_half_mirror
    if constexpr (LPK >= 16)
        x += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x140, 0xF, 0xF, false));  // row_mirror
    if constexpr (LPK == 32) x += __shfl_xor(x, 16, 64);
    return x;
}

typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 dec_bf16x2;

// q . k over the 8 components of a slice: bf16 pairs go straight into v_dot2 (exact products, fp32 sum)
__device__ inline float slice_dot(const Raw8<uint16_t>& q, const Raw8<uint16_t>& k)
{
    float d = 0.f;
    d = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(dec_bf16x2, q.u.x), __builtin_bit_cast(dec_bf16x2, k.u.x), d, false);
    d = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(dec_bf16x2, q.u.y), __builtin_bit_cast(dec_bf16x2, k.u.y), d, false);
    d = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(dec_bf16x2, q.u.z), __builtin_bit_cast(dec_bf16x2, k.u.z), d, false);
    d = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(dec_bf16x2, q.u.w), __builtin_bit_cast(dec_bf16x2, k.u.w), d, false);
    return d;
}
typedef __attribute__((__vector_size__(2 * sizeof(_Float16)))) _Float16 dec_f16x2;
__device__ inline float slice_dot(const Raw8<f16_bits>& q, const Raw8<f16_bits>& k)
{
    float d = 0.f;
    d = __builtin_amdgcn_fdot2(__builtin_bit_cast(dec_f16x2, q.u.x), __builtin_bit_cast(dec_f16x2, k.u.x), d, false);
    d = __builtin_amdgcn_fdot2(__builtin_bit_cast(dec_f16x2, q.u.y), __builtin_bit_cast(dec_f16x2, k.u.y), d, false);
    d = __builtin_amdgcn_fdot2(__builtin_bit_cast(dec_f16x2, q.u.z), __builtin_bit_cast(dec_f16x2, k.u.z), d, false);
    d = __builtin_amdgcn_fdot2(__builtin_bit_cast(dec_f16x2, q.u.w), __builtin_bit_cast(dec_f16x2, k.u.w), d, false);
    return d;
}
__device__ inline float slice_dot(const Raw8<float>& q, const Raw8<float>& k)
{
    float d = q.a.x * k.a.x;
    d = fmaf(q.a.y, k.a.y, d); d = fmaf(q.a.z, k.a.z, d); d = fmaf(q.a.w, k.a.w, d);
    d = fmaf(q.b.x, k.b.x, d); d = fmaf(q.b.y, k.b.y, d); d = fmaf(q.b.z, k.b.z, d); d = fmaf(q.b.w, k.b.w, d);
    return d;
}

constexpr float DEC_LOG2E = 1.4426950408889634f;

// Two ways to enumerate the keys below the window.  List mode walks the position lists of the query's groups
// (list entry -> position -> mask, two dependent loads per entry; a key that sits in several of the lists
// comes up once per list and is dropped from all but the first).  Scan mode walks the positions themselves and
// tests every key's mask against the query's (one coalesced load, consecutive K/V rows).  The lists win when
// they hold fewer entries than there are positions below the window; from there on the scan is the shorter walk.
__device__ inline bool decode_scan_mode(int list_entries, int below_window) { return list_entries >= below_window; }

// The walk of one work-group, in LDS.  List mode: segment 0 is the window, segment s > 0 the list prefix of one
// group; scan mode (nseg = 0): one run of pos + 1 positions.
struct DecWalk {
    int beg[34];              // first entry of every segment; beg[nseg] (beg[0] in scan mode) = entries in all
    int grp[33];              // group of the segment
    uint32_t prev[33];        // groups of the segments before it: a key that sits in one of them was taken there
    int nseg;
};

// One thread fills the walk for the groups in `groups` (of one query, or of all query heads of a KV head).
__device__ inline void decode_walk_init(DecWalk& W, uint32_t groups, const int* __restrict__ wptr, int K, int pos, int lo_w)
{
    int nseg = 1, run = pos - lo_w + 1;
    uint32_t prev = 0;
    W.beg[0] = 0; W.grp[0] = -1; W.prev[0] = 0;
    for (int g = 0; g < K; ++g) {
        if (!((groups >> g) & 1u)) continue;
        W.beg[nseg] = run; W.grp[nseg] = g; W.prev[nseg] = prev;
        run += wptr[g];                           // list entries below the window (kept by the route kernel)
        prev |= (1u << g);
        ++nseg;
    }
    W.beg[nseg] = run;
    W.nseg = nseg;
    if (decode_scan_mode(run - (pos - lo_w + 1), lo_w)) { W.nseg = 0; W.beg[0] = pos + 1; }
}

// Entry v of the walk -> cache row of its key, or -1 when no head attends it or an earlier segment had it;
// hb = the set of heads that attend it (bit i: the key's groups meet gq[i]; every head inside the window).
// single: every key sits in one group only (topk = 1), so a list entry's heads follow from its list's group and
// the key's mask is not read.
template <int NH>
__device__ inline int decode_walk_key(const DecWalk& W, int nseg, int v, int lo_w, const int* __restrict__ lists, int n,
                                      const uint32_t* __restrict__ mk, const uint32_t (&gq)[NH], uint32_t all_heads, bool single,
                                      uint32_t& hb)
{
    hb = 0;
    if (nseg == 0) {
        if (v >= lo_w) {
            hb = all_heads;
        } else {
            const uint32_t mkj = mk[v];
#pragma unroll
            for (int i = 0; i < NH; ++i) hb |= ((mkj & gq[i]) != 0u) ? (1u << i) : 0u;
        }
        return hb ? v : -1;
    }
    int sgi = 0;
    while (sgi + 1 < nseg && v >= W.beg[sgi + 1]) ++sgi;
    if (sgi == 0) {
        hb = all_heads;
        return lo_w + v;
    }
    const int j = lists[(size_t)W.grp[sgi] * n + (v - W.beg[sgi])];
    const uint32_t pv = W.prev[sgi];
    if (single) {
#pragma unroll
        for (int i = 0; i < NH; ++i) hb |= ((gq[i] >> W.grp[sgi]) & 1u) << i;
        return j;
    }
    if (NH == 1) {                                // the key is in a group of the one query: only the dedup needs its mask
        hb = 1u;
        return (pv != 0u && (mk[j] & pv) != 0u) ? -1 : j;
    }
    const uint32_t mkj = mk[j];
    if ((mkj & pv) != 0u) return -1;
#pragma unroll
    for (int i = 0; i < NH; ++i) hb |= ((mkj & gq[i]) != 0u) ? (1u << i) : 0u;
    return j;
}

// A chunk of the walk for the grouped-query kernels (256 threads): every thread resolves KPT entries (all loads
// independent), then the skipped ones are squeezed out: wave ballots give every (pass, wavefront) its count, the
// kept keys land in pass-major, wavefront-major order in s_j / s_hb, padded with -1 / 0 up to `cap` entries.
// Returns the number of keys kept.  Two barriers inside.
template <int KPT, int NH, typename HB>
__device__ inline int decode_resolve_chunk(const DecWalk& W, int nseg, int v0, int nk0, int lo_w, const int* __restrict__ lists, int n,
                                           const uint32_t* __restrict__ mk, const uint32_t (&gq)[NH], uint32_t all_heads, bool single,
                                           int* s_j, HB* s_hb, int cap, int* s_wcnt)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    int js[KPT];
    uint32_t hbv[KPT];
#pragma unroll
    for (int it = 0; it < KPT; ++it) {
        js[it] = -1;
        hbv[it] = 0;
        const int i0 = it * 256 + tid;
        if (i0 < nk0) js[it] = decode_walk_key<NH>(W, nseg, v0 + i0, lo_w, lists, n, mk, gq, all_heads, single, hbv[it]);
    }
    unsigned long long bal[KPT];
#pragma unroll
    for (int it = 0; it < KPT; ++it) {
        bal[it] = __ballot(js[it] >= 0);
        if (lane == 0) s_wcnt[it * 4 + wave] = __popcll(bal[it]);
    }
    for (int i = tid; i < cap; i += 256) { s_j[i] = -1; s_hb[i] = 0; }
    __syncthreads();
    int nk = 0;
#pragma unroll
    for (int it = 0; it < KPT; ++it) {
        int before = 0;
        for (int w2 = 0; w2 < it * 4 + wave; ++w2) before += s_wcnt[w2];
        if (js[it] >= 0) {
            const unsigned long long lt = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
            const int dst = before + __popcll(bal[it] & lt);
            s_j[dst] = js[it];
            s_hb[dst] = (HB)hbv[it];
        }
    }
#pragma unroll
    for (int w2 = 0; w2 < 4 * KPT; ++w2) nk += s_wcnt[w2];
    __syncthreads();
    return nk;
}

template <typename T, int D>
__global__ __launch_bounds__(256) void decode_attn_kernel(DecodeLayout L, HeadMap hm, int pos_arg, const int* __restrict__ pos_dev, int span,
                                                          const T* __restrict__ q_new,
                                                          const T* __restrict__ kc, const T* __restrict__ vc,
                                                          const char* __restrict__ st, float* __restrict__ part)
{
    constexpr int LPK = lanes_per_key(D);         // lanes that share one key (8 components each)
    constexpr int ACT = D / 8;                    // ... of which this many hold components (all, unless d is 80 or 96)
    constexpr int SLOTS = 64 / LPK;               // keys a wavefront handles side by side
    constexpr int PW = D + 4;                     // floats of one partial: o[D], max (log2 units), sum, count
    constexpr int U = sizeof(T) == 2 ? 8 : 4;     // keys in flight per slice: U K rows and U V rows loaded before use
    __shared__ DecWalk s_walk;
    __shared__ int s_j[DEC_CHUNK];                // cache row of every key of the chunk, -1 = skipped
    __shared__ float s_red[4][SLOTS][PW];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int slot = lane / LPK, sub = lane % LPK;
    const int chunk = blockIdx.x, bhq = blockIdx.y;
    const int b = bhq / L.Hq, h = bhq % L.Hq;
    const int pos = pos_dev ? pos_dev[b] : pos_arg;
    if (pos < 0 || pos >= L.n) return;
    const size_t bhk = (size_t)b * L.Hkv + hm.kv[h];
    const int lo_w = max(0, pos - L.window + 1);  // first position of the window
    const uint32_t gq = ((const uint32_t*)(st + L.off_mq))[bhq];
    const int* wptr = (const int*)(st + L.off_wp) + bhk * L.K;
    const int* lists = (const int*)(st + L.off_lists) + bhk * L.K * L.n;
    const uint32_t* mk = (const uint32_t*)(st + L.off_mk) + bhk * L.n;

    if (tid == 0) decode_walk_init(s_walk, gq, wptr, L.K, pos, lo_w);
    __syncthreads();
    const int nseg = s_walk.nseg;
    const int vtotal = s_walk.beg[nseg];
    const uint32_t gq1[1] = {gq};
    float* mypart = part + ((size_t)bhq * L.max_parts + chunk) * PW;
    if ((long)chunk * DEC_CHUNK >= vtotal) {     // nothing for this work-group
        for (int e = tid; e < PW; e += 256) mypart[e] = (e == D) ? -INFINITY : 0.f;
        return;
    }
    const bool act = (ACT == LPK) || sub < ACT;
    Raw8<T> qr;
    if (act) qr.load(q_new + (size_t)bhq * D + sub * 8); else qr.zero();
    float o[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) o[e] = 0.f;
    float m = -INFINITY, l = 0.f;                 // running max in log2 units, running sum
    int cnt = 0;
    const float sl2 = L.scale * DEC_LOG2E, cap = L.softcap;
    const T* kbase = kc + bhk * L.n * D + sub * 8;
    const T* vbase = vc + bhk * L.n * D + sub * 8;

    // rounds of SLOTS*U keys per wavefront, the 4 wavefronts interleaved; one softmax update per round
    for (int cc = 0; cc < span; ++cc) {
    // chunks chunk, chunk + gridDim.x, ...: however short the walk turns out, its chunks spread over the work-groups
    const long v0l = ((long)chunk + (long)cc * gridDim.x) * DEC_CHUNK;
    if (v0l >= vtotal) break;                      // uniform over the work-group
    const int v0 = (int)v0l;
    if (cc > 0) __syncthreads();                  // the last chunk's rows have been read
    // resolve the whole chunk at once: list entry -> position -> (mask check); all loads independent
    const int nk = min(vtotal - v0, DEC_CHUNK);
    for (int i = tid; i < DEC_CHUNK; i += 256) {
        int j = -1;
        uint32_t hb;
        if (i < nk) j = decode_walk_key<1>(s_walk, nseg, v0 + i, lo_w, lists, L.n, mk, gq1, 1u, L.topk == 1, hb);
        s_j[i] = j;
    }
    __syncthreads();

    for (int r0 = wave * (SLOTS * U); r0 < nk; r0 += 4 * SLOTS * U) {
        int jpos[U];
        Raw8<T> kr[U], vr[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            jpos[u] = s_j[r0 + u * SLOTS + slot];                     // r0 + U*SLOTS <= DEC_CHUNK: in bounds
            const int j = max(jpos[u], 0);
            if (act) { kr[u].load(kbase + (size_t)j * D); vr[u].load(vbase + (size_t)j * D); }
            else { kr[u].zero(); vr[u].zero(); }
        }
        float xs[U];
        float mx = -INFINITY;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const float dot = slice_sum<LPK>(slice_dot(qr, kr[u]));
            float x = dot * sl2;
            if (cap > 0.f) x = cap * DEC_LOG2E * tanhf(dot * L.scale / cap);
            xs[u] = (jpos[u] < 0) ? -INFINITY : x;
            mx = fmaxf(mx, xs[u]);
            cnt += (jpos[u] < 0) ? 0 : 1;
        }
        const float m_new = fmaxf(m, mx);
        if (m_new == -INFINITY) continue;         // nothing attended so far (uniform over the slice)
        const float alpha = __builtin_amdgcn_exp2f(m - m_new);        // m = -inf: 0
        m = m_new;
        l *= alpha;
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] *= alpha;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const float pr = __builtin_amdgcn_exp2f(xs[u] - m_new);   // skipped keys: exp2(-inf) = 0
            float vx[8];
            vr[u].unpack(vx);
            l += pr;
#pragma unroll
            for (int e = 0; e < 8; ++e) o[e] = fmaf(pr, vx[e], o[e]);
        }
    }
    }   // chunks of the span
    // every (wavefront, slot) holds a partial softmax over its keys: fold them through LDS
    {
        float* r = s_red[wave][slot];
        if (act) {
#pragma unroll
            for (int e = 0; e < 8; ++e) r[sub * 8 + e] = o[e];
        }
        if (sub == 0) { r[D] = m; r[D + 1] = l; r[D + 2] = (float)cnt; }
    }
    __syncthreads();
    if (tid < D) {
        float mx = -INFINITY;
        for (int w2 = 0; w2 < 4; ++w2)
            for (int s2 = 0; s2 < SLOTS; ++s2) mx = fmaxf(mx, s_red[w2][s2][D]);
        float acc = 0.f, lsum = 0.f, csum = 0.f;
        for (int w2 = 0; w2 < 4; ++w2)
            for (int s2 = 0; s2 < SLOTS; ++s2) {
                const float ms = s_red[w2][s2][D];
                const float wgt = (ms == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(ms - mx);
                acc += wgt * s_red[w2][s2][tid];
                lsum += wgt * s_red[w2][s2][D + 1];
                csum += s_red[w2][s2][D + 2];
            }
        mypart[tid] = acc;
        if (tid == 0) { mypart[D] = mx; mypart[D + 1] = lsum; mypart[D + 2] = csum; mypart[D + 3] = 0.f; }
    }
}

// ---------------------------------------------------------------- step 2, grouped-query form
// The G query heads of one KV head read the same K and V rows, so one work-group serves all of them:
// the key sequence is the window plus the list prefixes of the UNION of the heads' groups (a key is
// taken from the first of those groups it belongs to), every key carries the set of heads that attend
// it (window: all; list key: the heads whose groups meet the key's), and each K/V row is loaded once
// for G softmaxes.  Keys skipped by the dedup are squeezed out of the chunk before the arithmetic.
// Requires the default head map (query heads hk*G .. hk*G+G-1 belong to KV head hk).
template <typename T, int D, int G>
__global__ __launch_bounds__(256) void decode_attn_gqa_kernel(DecodeLayout L, int pos_arg, const int* __restrict__ pos_dev, int span,
                                                              const T* __restrict__ q_new,
                                                              const T* __restrict__ kc, const T* __restrict__ vc,
                                                              const char* __restrict__ st, float* __restrict__ part)
{
    constexpr int LPK = lanes_per_key(D);
    constexpr int ACT = D / 8;
    constexpr int SLOTS = 64 / LPK;
    constexpr int PW = D + 4;
    constexpr int U = (G <= 2 && sizeof(T) == 2) ? 8 : 4;    // keys per slot and round: U K rows and U V rows in flight
    constexpr int KPT = DEC_CHUNK / 256;                     // keys every thread resolves per chunk
    constexpr int HB = G < 4 ? G : 4;                        // heads folded through LDS at a time
    __shared__ DecWalk s_walk;
    __shared__ int s_j[DEC_CHUNK + 4 * SLOTS * U];    // cache rows of the chunk's keys, squeezed; padded with -1
    __shared__ uint8_t s_hb[DEC_CHUNK + 4 * SLOTS * U];   // which of the G heads attend the key
    __shared__ int s_wcnt[4 * KPT];
    __shared__ float s_red[HB][4 * SLOTS][PW];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int slot = lane / LPK, sub = lane % LPK;
    const int chunk = blockIdx.x;
    const size_t bhk = blockIdx.y;
    const int b = (int)(bhk / L.Hkv), hk = (int)(bhk % L.Hkv);
    const int pos = pos_dev ? pos_dev[b] : pos_arg;
    if (pos < 0 || pos >= L.n) return;
    const size_t bhq0 = (size_t)b * L.Hq + (size_t)hk * G;
    const int lo_w = max(0, pos - L.window + 1);
    uint32_t gq[G];
    uint32_t gu = 0;
#pragma unroll
    for (int i = 0; i < G; ++i) { gq[i] = ((const uint32_t*)(st + L.off_mq))[bhq0 + i]; gu |= gq[i]; }
    const int* wptr = (const int*)(st + L.off_wp) + bhk * L.K;
    const int* lists = (const int*)(st + L.off_lists) + bhk * L.K * L.n;
    const uint32_t* mk = (const uint32_t*)(st + L.off_mk) + bhk * L.n;

    if (tid == 0) decode_walk_init(s_walk, gu, wptr, L.K, pos, lo_w);
    __syncthreads();
    const int nseg = s_walk.nseg;
    const int vtotal = s_walk.beg[nseg];
    // this work-group walks up to `span` chunks of the sequence, gridDim.x apart, and leaves one partial per head
    if ((long)chunk * DEC_CHUNK >= vtotal) {
        for (int i = 0; i < G; ++i) {
            float* mypart = part + ((bhq0 + i) * L.max_parts + chunk) * PW;
            for (int e = tid; e < PW; e += 256) mypart[e] = (e == D) ? -INFINITY : 0.f;
        }
        return;
    }
    const bool act = (ACT == LPK) || sub < ACT;
    Raw8<T> qr[G];
#pragma unroll
    for (int i = 0; i < G; ++i) {
        if (act) qr[i].load(q_new + (bhq0 + i) * D + sub * 8); else qr[i].zero();
    }
    float o[G][8], m[G], l[G];
    int cnt[G];
#pragma unroll
    for (int i = 0; i < G; ++i) {
        m[i] = -INFINITY; l[i] = 0.f; cnt[i] = 0;
#pragma unroll
        for (int e = 0; e < 8; ++e) o[i][e] = 0.f;
    }
    const float sl2 = L.scale * DEC_LOG2E, cap = L.softcap;
    const T* kbase = kc + bhk * L.n * D + (act ? sub * 8 : 0);
    const T* vbase = vc + bhk * L.n * D + (act ? sub * 8 : 0);

    // one round: U keys per slot.  `fetch` issues the K and V row loads of a round, `fold` does its arithmetic.
    struct Round {
        int jpos[U];
        uint32_t hbs[U];
        Raw8<T> kr[U], vr[U];
    };
    auto fetch = [&](Round& R, int r0) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            R.jpos[u] = s_j[r0 + u * SLOTS + slot];                   // the array is padded by one round of -1
            R.hbs[u] = (R.jpos[u] >= 0) ? (uint32_t)s_hb[r0 + u * SLOTS + slot] : 0u;
            const int j = max(R.jpos[u], 0);
            // lanes past d / 8 slices (d = 80, 96) read the row's first slice again: their q is zero and their
            // output is never stored
            R.kr[u].load(kbase + (size_t)j * D);
            R.vr[u].load(vbase + (size_t)j * D);
        }
    };
    auto fold = [&](const Round& R) {
        float vx[U][8];
#pragma unroll
        for (int u = 0; u < U; ++u) R.vr[u].unpack(vx[u]);
        uint32_t hb_or = 0;
#pragma unroll
        for (int u = 0; u < U; ++u) hb_or |= R.hbs[u];
#pragma unroll
        for (int i = 0; i < G; ++i) {
            // a list segment holds the keys of one group: with few groups per key most heads want none of
            // the keys of a round, and the whole wavefront skips them
            if (!__any((hb_or >> i) & 1u)) continue;
            float xs[U];
            float mx = -INFINITY;
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const float dot = slice_sum<LPK>(slice_dot(qr[i], R.kr[u]));
                float x = dot * sl2;
                if (cap > 0.f) x = cap * DEC_LOG2E * tanhf(dot * L.scale / cap);
                const bool on = (R.hbs[u] >> i) & 1u;
                xs[u] = on ? x : -INFINITY;
                mx = fmaxf(mx, xs[u]);
                cnt[i] += on ? 1 : 0;
            }
            const float m_new = fmaxf(m[i], mx);
            if (m_new != -INFINITY) {
                const float alpha = __builtin_amdgcn_exp2f(m[i] - m_new);
                m[i] = m_new;
                l[i] *= alpha;
#pragma unroll
                for (int e = 0; e < 8; ++e) o[i][e] *= alpha;
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const float pr = __builtin_amdgcn_exp2f(xs[u] - m_new);
                    l[i] += pr;
#pragma unroll
                    for (int e = 0; e < 8; ++e) o[i][e] = fmaf(pr, vx[u][e], o[i][e]);
                }
            }
        }
    };

    for (int cc = 0; cc < span; ++cc) {
    // chunks chunk, chunk + gridDim.x, ...: however short the walk turns out, its chunks spread over the work-groups
    const long v0l = ((long)chunk + (long)cc * gridDim.x) * DEC_CHUNK;
    if (v0l >= vtotal) break;                      // uniform over the work-group
    const int v0 = (int)v0l;
    if (cc > 0) __syncthreads();                  // the last chunk's rows have been read
    const int nk = decode_resolve_chunk<KPT, G, uint8_t>(s_walk, nseg, v0, min(vtotal - v0, DEC_CHUNK), lo_w, lists, L.n, mk, gq,
                                                (1u << G) - 1u, L.topk == 1, s_j, s_hb, DEC_CHUNK + 4 * SLOTS * U, s_wcnt);
    constexpr int RSTEP = 4 * SLOTS * U;          // keys of one round of the four wavefronts
    // (Keeping the loads of the next round in flight while this one is folded costs a second set of row
    // registers and a wavefront of occupancy: slower at every context length measured.)
    for (int r0 = wave * (SLOTS * U); r0 < nk; r0 += RSTEP) {
        Round ra;
        fetch(ra, r0);
        fold(ra);
    }
    }   // chunks of the span
    // fold the (wavefront, slot) partials through LDS, HB heads at a time: 256 / HB threads per head
    constexpr int TPH = 256 / HB;
    const int hsel = tid / TPH, t = tid % TPH;
#pragma unroll
    for (int h0 = 0; h0 < G; h0 += HB) {
        if (h0 > 0) __syncthreads();
#pragma unroll
        for (int ii = 0; ii < HB; ++ii) {
            const int i = h0 + ii;
            float* r = s_red[ii][wave * SLOTS + slot];
            if (act) {
#pragma unroll
                for (int e = 0; e < 8; ++e) r[sub * 8 + e] = o[i][e];
            }
            if (sub == 0) { r[D] = m[i]; r[D + 1] = l[i]; r[D + 2] = (float)cnt[i]; }
        }
        __syncthreads();
        {
            const float (*rr)[PW] = s_red[hsel];
            float mx = -INFINITY;
#pragma unroll
            for (int s2 = 0; s2 < 4 * SLOTS; ++s2) mx = fmaxf(mx, rr[s2][D]);
            float wgt[4 * SLOTS];
            float lsum = 0.f, csum = 0.f;
#pragma unroll
            for (int s2 = 0; s2 < 4 * SLOTS; ++s2) {
                const float ms = rr[s2][D];
                wgt[s2] = (ms == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(ms - mx);
                lsum += wgt[s2] * rr[s2][D + 1];
                csum += rr[s2][D + 2];
            }
            float* mypart = part + ((bhq0 + h0 + hsel) * L.max_parts + chunk) * PW;
            for (int c = t; c < D; c += TPH) {
                float acc = 0.f;
#pragma unroll
                for (int s2 = 0; s2 < 4 * SLOTS; ++s2) acc += wgt[s2] * rr[s2][c];
                mypart[c] = acc;
            }
            if (t == 0) { mypart[D] = mx; mypart[D + 1] = lsum; mypart[D + 2] = csum; mypart[D + 3] = 0.f; }
        }
    }
}

// ---------------------------------------------------------------- step 2, grouped-query form on the matrix cores
// The same walk as decode_attn_gqa_kernel for 16-bit caches, with both products on
// v_mfma_f32_16x16x32: a wavefront takes 32 keys per round as two blocks of 16.
//   S^T[key, head] = K[key, :] . Q[head, :]   A = K rows straight from the cache (lane: key l%16, components
//                                             32*kb + 8*(l/16) ..+8, one 16-byte load per product), B = the G <= 16
//                                             query heads of the KV head (columns past G are zero);
//   the accumulator lane (head l%16, keys 4*(l/16) ..+4 of either block) does the softmax step of its head;
//   its 8 probabilities, rounded to 16 bits, ARE the B operand of
//   O^T[c, head] += V^T[c, key] P^T[key, head]  A = 16 components x 32 keys of V^T.
// V^T is not in memory: the V rows of the round land in LDS by global_load_lds (no registers), and each lane
// picks the 8 keys of its k-slice for its component with 16-bit LDS reads.  The rows of one wave load sit
// 1 KB + 32 bytes apart from the next load's, so the four keys the lane groups read together fall on
// different banks.  The softmax reference moves only when the maximum has drifted by more than 8 (log2
// units), so the accumulators are rarely rescaled.
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 dec_bf16x8;
typedef __attribute__((__vector_size__(8 * sizeof(_Float16)))) _Float16 dec_f16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float dec_f32x4;
typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t dec_u32x4;

template <bool F16> struct DecHalf;
template <> struct DecHalf<false> {
    typedef dec_bf16x8 V8;
    static __device__ inline dec_f32x4 mfma(V8 a, V8 b, dec_f32x4 c) { return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0); }
    static __device__ inline uint32_t pack2(float lo, float hi, float& sum)
    {
        const __bf16 a = (__bf16)lo, b = (__bf16)hi;
        sum += (float)a + (float)b;
        return (uint32_t)__builtin_bit_cast(uint16_t, a) | ((uint32_t)__builtin_bit_cast(uint16_t, b) << 16);
    }
};
template <> struct DecHalf<true> {
    typedef dec_f16x8 V8;
    static __device__ inline dec_f32x4 mfma(V8 a, V8 b, dec_f32x4 c) { return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0); }
    static __device__ inline uint32_t pack2(float lo, float hi, float& sum)
    {
        const _Float16 a = (_Float16)lo, b = (_Float16)hi;
        sum += (float)a + (float)b;
        return (uint32_t)__builtin_bit_cast(uint16_t, a) | ((uint32_t)__builtin_bit_cast(uint16_t, b) << 16);
    }
};

constexpr float DEC_RESCALE_THRESHOLD = 8.f;

// CH: entries of the walk a work-group resolves at a time (the long or the short chunk: the short one when the
// launch would otherwise leave most of the chip idle, one round per wavefront and four times the work-groups).
template <bool F16, int D, int CH>
__global__ __launch_bounds__(256) void decode_attn_gqa_mfma_kernel(DecodeLayout L, int Gall, int pos_arg, const int* __restrict__ pos_dev,
                                                                   int span, const uint16_t* __restrict__ q_new,
                                                                   const uint16_t* __restrict__ kc, const uint16_t* __restrict__ vc,
                                                                   const char* __restrict__ st, float* __restrict__ part)
{
    typedef DecHalf<F16> HT;
    typedef typename HT::V8 V8;
    static_assert(D % 16 == 0 && D >= 64 && D <= 256, "whole 16-component blocks");
    constexpr int RB = D * 2;                     // bytes of a cache row
    constexpr int LPR = RB / 16;                  // lanes that load one V row (8, 10, 12, 16, 32)
    constexpr int RPI = 64 / LPR;                 // whole V rows per wave load (the lanes past RPI * LPR repeat lane 0)
    constexpr int NI = (32 + RPI - 1) / RPI;      // wave loads per round of 32 keys
    constexpr int IPITCH = 1024 + 32;             // LDS bytes from one wave load to the next
    constexpr int VBYTES = NI * IPITCH;           // V rows of a round, per wavefront
    constexpr int KB = (D + 31) / 32;             // products of one S^T block (the last one partly zero for d = 80)
    constexpr int NB = D / 16;                    // 16-component blocks of O^T
    constexpr int PW = D + 4;
    constexpr int KPT = CH >= 256 ? CH / 256 : 1;
    constexpr int RSTEP = 4 * 32;                 // keys of one round of the four wavefronts
    constexpr int GMAX = 16;                      // query heads per work-group: the columns of the products
    constexpr int RED_BYTES = GMAX * 4 * PW * 4;
    constexpr int BUF_BYTES = 4 * VBYTES > RED_BYTES ? 4 * VBYTES : RED_BYTES;
    __shared__ DecWalk s_walk;
    __shared__ int s_j[CH + RSTEP];        // cache rows of the chunk's keys, squeezed; padded with -1
    __shared__ __attribute__((aligned(8))) uint16_t s_hb[CH + RSTEP];  // which heads attend the key; 0 in the padding
    __shared__ int s_wcnt[4 * KPT];
    __shared__ __attribute__((aligned(16))) char s_buf[BUF_BYTES];   // V rows of the rounds; the partials at the end

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int m16 = lane & 15, qg = lane >> 4;
    const int chunk = blockIdx.x;
    // more than GMAX query heads per KV head (Gall): the heads go in sub-groups of GMAX, one work-group row each
    const int nsub = (Gall + GMAX - 1) / GMAX;
    const size_t bhk = blockIdx.y / nsub;
    const int sub = (int)(blockIdx.y % nsub);
    const int G = min(GMAX, Gall - sub * GMAX);
    const int b = (int)(bhk / L.Hkv), hk = (int)(bhk % L.Hkv);
    const int pos = pos_dev ? pos_dev[b] : pos_arg;
    if (pos < 0 || pos >= L.n) return;
    const size_t bhq0 = (size_t)b * L.Hq + (size_t)hk * Gall + (size_t)sub * GMAX;
    const int lo_w = max(0, pos - L.window + 1);
    uint32_t gq[GMAX];
    uint32_t gu = 0;
#pragma unroll
    for (int i = 0; i < GMAX; ++i) { gq[i] = (i < G) ? ((const uint32_t*)(st + L.off_mq))[bhq0 + i] : 0u; gu |= gq[i]; }
    const int* wptr = (const int*)(st + L.off_wp) + bhk * L.K;
    const int* lists = (const int*)(st + L.off_lists) + bhk * L.K * L.n;
    const uint32_t* mk = (const uint32_t*)(st + L.off_mk) + bhk * L.n;

    if (tid == 0) decode_walk_init(s_walk, gu, wptr, L.K, pos, lo_w);
    __syncthreads();
    const int nseg = s_walk.nseg;
    const int vtotal = s_walk.beg[nseg];
    if ((long)chunk * CH >= vtotal) {
        for (int i = 0; i < G; ++i) {
            float* mypart = part + ((bhq0 + i) * L.max_parts + chunk) * PW;
            for (int e = tid; e < PW; e += 256) mypart[e] = (e == D) ? -INFINITY : 0.f;
        }
        return;
    }
    // B operand of S^T: the query heads, column m16 (zero past G)
    V8 qv[KB];
#pragma unroll
    for (int kb = 0; kb < KB; ++kb) {
        dec_u32x4 w = {0u, 0u, 0u, 0u};
        if (m16 < G && 32 * kb + 8 * qg < D) w = *(const dec_u32x4*)(q_new + (bhq0 + m16) * D + 32 * kb + 8 * qg);
        qv[kb] = __builtin_bit_cast(V8, w);
    }
    dec_f32x4 oacc[NB];
#pragma unroll
    for (int blk = 0; blk < NB; ++blk) oacc[blk] = dec_f32x4{0.f, 0.f, 0.f, 0.f};
    float m_ref = -INFINITY, lsum = 0.f;          // of head m16, over the keys of this lane group so far
    int cnt = 0;
    const float sl2 = L.scale * DEC_LOG2E, cap = L.softcap;
    const uint16_t* kbase = kc + bhk * L.n * D + 8 * qg;
    const uint16_t* vbase = vc + bhk * L.n * D;
    const unsigned lds_v = lds_addr_of(&s_buf[0]) + (unsigned)wave * VBYTES;
    const int dlane = (lane < RPI * LPR) ? lane : 0;                  // the lane whose row chunk this lane loads
    const char* my_v = s_buf + wave * VBYTES;
    // k-slot e of lane group qg holds key 16*(e/4) + 4*qg + e%4 of the round: LDS offset of that key's V row
    int vrow[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const int key = 16 * (e / 4) + 4 * qg + e % 4;
        vrow[e] = (key / RPI) * IPITCH + (key % RPI) * RB + 2 * m16;
    }

    for (int cc = 0; cc < span; ++cc) {
    // chunks chunk, chunk + gridDim.x, ...: however short the walk turns out, its chunks spread over the work-groups
    const long v0l = ((long)chunk + (long)cc * gridDim.x) * CH;
    if (v0l >= vtotal) break;                      // uniform over the work-group
    const int v0 = (int)v0l;
    if (cc > 0) __syncthreads();                  // the last chunk's keys have been read
    const int nk = decode_resolve_chunk<KPT, GMAX, uint16_t>(s_walk, nseg, v0, min(vtotal - v0, CH), lo_w, lists, L.n, mk, gq,
                                                             (1u << G) - 1u, L.topk == 1, s_j, s_hb, CH + RSTEP, s_wcnt);

    for (int r0 = wave * 32; r0 < nk; r0 += RSTEP) {
        // the V rows of the round -> LDS (wave load i holds keys i*RPI ..+RPI of the round)
        // (a wave load past the 32nd key fetches rows of the next round or row 0: read by nobody)
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const int jv = max(s_j[r0 + i * RPI + dlane / LPR], 0);
            lds_dma16(vbase, (unsigned)jv * (unsigned)RB + (unsigned)(dlane % LPR) * 16u, lds_v + i * IPITCH);
        }
        // the K rows of the two blocks -> registers
        const int ja = max(s_j[r0 + m16], 0), jb = max(s_j[r0 + 16 + m16], 0);
        V8 ka[KB], kb2[KB];
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) {
            dec_u32x4 wa = {0u, 0u, 0u, 0u}, wb = {0u, 0u, 0u, 0u};
            if (32 * kb + 8 * qg < D) {                               // false only in the last product of d = 80
                wa = *(const dec_u32x4*)(kbase + (size_t)ja * D + 32 * kb);
                wb = *(const dec_u32x4*)(kbase + (size_t)jb * D + 32 * kb);
            }
            ka[kb] = __builtin_bit_cast(V8, wa);
            kb2[kb] = __builtin_bit_cast(V8, wb);
        }
        const uint64_t hba = *(const uint64_t*)(&s_hb[r0 + 4 * qg]);           // 16 head bits for each of the four keys
        const uint64_t hbb = *(const uint64_t*)(&s_hb[r0 + 16 + 4 * qg]);
        dec_f32x4 sa = {0.f, 0.f, 0.f, 0.f}, sb = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) {
            sa = HT::mfma(ka[kb], qv[kb], sa);
            sb = HT::mfma(kb2[kb], qv[kb], sb);
        }
        float x[8];
        float mloc = -INFINITY;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float sc = (e < 4) ? sa[e % 4] : sb[e % 4];
            const uint32_t heads = (uint32_t)(((e < 4) ? hba : hbb) >> (16 * (e % 4))) & 0xffffu;
            const bool on = (heads >> m16) & 1u;
            float xv = sc * sl2;
            if (cap > 0.f) xv = cap * DEC_LOG2E * tanhf(sc * L.scale / cap);
            x[e] = on ? xv : -INFINITY;
            mloc = fmaxf(mloc, x[e]);
            cnt += on ? 1 : 0;
        }
        mloc = fmaxf(mloc, __shfl_xor(mloc, 16, 64));
        mloc = fmaxf(mloc, __shfl_xor(mloc, 32, 64));
        const bool move = mloc > m_ref + DEC_RESCALE_THRESHOLD;       // also true for the first attended key (m_ref = -inf)
        if (__any(move)) {
            const float m_new = move ? mloc : m_ref;
            const float alpha = (m_ref == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(m_ref - m_new);
            m_ref = m_new;
            lsum *= alpha;
#pragma unroll
            for (int blk = 0; blk < NB; ++blk) oacc[blk] *= alpha;
        }
        const float mr = (m_ref == -INFINITY) ? 0.f : m_ref;
        dec_u32x4 pw;
        float psum = 0.f;
#pragma unroll
        for (int e2 = 0; e2 < 4; ++e2)
            pw[e2] = HT::pack2(__builtin_amdgcn_exp2f(x[2 * e2] - mr), __builtin_amdgcn_exp2f(x[2 * e2 + 1] - mr), psum);
        lsum += psum;
        const V8 pb = __builtin_bit_cast(V8, pw);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");              // the V rows have landed
#pragma unroll
        for (int blk = 0; blk < NB; ++blk) {
            dec_u32x4 vw;
#pragma unroll
            for (int e2 = 0; e2 < 4; ++e2) {
                const uint32_t lo = *(const uint16_t*)(my_v + vrow[2 * e2] + 32 * blk);
                const uint32_t hi = *(const uint16_t*)(my_v + vrow[2 * e2 + 1] + 32 * blk);
                vw[e2] = lo | (hi << 16);
            }
            oacc[blk] = HT::mfma(__builtin_bit_cast(V8, vw), pb, oacc[blk]);
        }
        asm volatile("" ::: "memory");                                // the reads stay ahead of the next round's loads
    }
    }   // chunks of the span
    // the lane groups of a head share the reference; their sums and counts add up
    lsum += __shfl_xor(lsum, 16, 64); lsum += __shfl_xor(lsum, 32, 64);
    cnt += __shfl_xor(cnt, 16, 64); cnt += __shfl_xor(cnt, 32, 64);
    __syncthreads();                              // every wavefront is done with its V rows
    float (*red)[4][PW] = (float (*)[4][PW])s_buf;
    if (m16 < G) {
        float* r = red[m16][wave];
#pragma unroll
        for (int blk = 0; blk < NB; ++blk)
#pragma unroll
            for (int e = 0; e < 4; ++e) r[16 * blk + 4 * qg + e] = oacc[blk][e];
        if (qg == 0) { r[D] = m_ref; r[D + 1] = lsum; r[D + 2] = (float)cnt; }
    }
    __syncthreads();
    {
        const int hsel = tid >> 4, t = tid & 15;  // 16 threads per head
        if (hsel < G) {
            const float (*rr)[PW] = red[hsel];
            float mx = -INFINITY;
#pragma unroll
            for (int w2 = 0; w2 < 4; ++w2) mx = fmaxf(mx, rr[w2][D]);
            float wgt[4];
            float ls = 0.f, cs = 0.f;
#pragma unroll
            for (int w2 = 0; w2 < 4; ++w2) {
                const float ms = rr[w2][D];
                wgt[w2] = (ms == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(ms - mx);
                ls += wgt[w2] * rr[w2][D + 1];
                cs += rr[w2][D + 2];
            }
            float* mypart = part + ((bhq0 + hsel) * L.max_parts + chunk) * PW;
            for (int c = t; c < D; c += 16) {
                float acc = 0.f;
#pragma unroll
                for (int w2 = 0; w2 < 4; ++w2) acc += wgt[w2] * rr[w2][c];
                mypart[c] = acc;
            }
            if (t == 0) { mypart[D] = mx; mypart[D + 1] = ls; mypart[D + 2] = cs; mypart[D + 3] = 0.f; }
        }
    }
}

// ---------------------------------------------------------------- step 3: merge of the chunks
// One work-group per (batch, query head).  A chunk's partial is read by D/4 threads (4 components each);
// the 256 / (D/4) groups of threads take the chunks round-robin, then fold through LDS.
template <typename T, int D>
__global__ __launch_bounds__(256) void decode_merge_kernel(DecodeLayout L, int pos_arg, const int* __restrict__ pos_dev, int nchunks,
                                                           const float* __restrict__ part,
                                                           T* __restrict__ out, float* __restrict__ lse,
                                                           int32_t* __restrict__ row_pairs)
{
    constexpr int PW = D + 4;
    constexpr int TPG = D / 4;                    // threads per group
    constexpr int NG = 256 / TPG;                 // whole groups; the threads past NG * TPG (d = 80, 96) idle
    __shared__ float s_acc[NG][D + 4];
    const int tid = threadIdx.x, t = tid % TPG, grp = tid / TPG, bhq = blockIdx.x;
    const int pos = pos_dev ? pos_dev[bhq / L.Hq] : pos_arg;
    if (pos < 0 || pos >= L.n) return;                // the other kernels of the step skipped this sequence too
    const float* p0 = part + (size_t)bhq * L.max_parts * PW;
    // every group of threads folds its share of the partials against a running maximum of its own (one pass over
    // the partials, four of them in flight per group); the groups then meet in LDS
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    float mrun = -INFINITY, lsum = 0.f, csum = 0.f;
    constexpr int MU = 4;
    for (int c0 = grp; grp < NG && c0 < nchunks; c0 += NG * MU) {
        float4 tail[MU], ov[MU];
#pragma unroll
        for (int u = 0; u < MU; ++u) {
            const int c = min(c0 + u * NG, nchunks - 1);              // clamped loads, skipped below
            const float* p = p0 + (size_t)c * PW;
            tail[u] = *(const float4*)(p + D);                        // max (log2 units), sum, count, unused
            ov[u] = *(const float4*)(p + 4 * t);
        }
        float mnew = mrun;
#pragma unroll
        for (int u = 0; u < MU; ++u)
            if (c0 + u * NG < nchunks) mnew = fmaxf(mnew, tail[u].x);
        if (mnew == -INFINITY) continue;                              // nothing attended so far
        const float alpha = __builtin_amdgcn_exp2f(mrun - mnew);      // mrun = -inf: 0
        mrun = mnew;
        acc.x *= alpha; acc.y *= alpha; acc.z *= alpha; acc.w *= alpha;
        lsum *= alpha;
#pragma unroll
        for (int u = 0; u < MU; ++u) {
            if (c0 + u * NG >= nchunks || tail[u].x == -INFINITY) continue;
            const float wgt = __builtin_amdgcn_exp2f(tail[u].x - mnew);
            acc.x = fmaf(wgt, ov[u].x, acc.x); acc.y = fmaf(wgt, ov[u].y, acc.y);
            acc.z = fmaf(wgt, ov[u].z, acc.z); acc.w = fmaf(wgt, ov[u].w, acc.w);
            lsum = fmaf(wgt, tail[u].y, lsum);
            csum += tail[u].z;
        }
    }
    if (grp < NG) {
        *(float4*)(&s_acc[grp][4 * t]) = acc;
        if (t == 0) { s_acc[grp][D] = lsum; s_acc[grp][D + 1] = csum; s_acc[grp][D + 2] = mrun; }
    }
    __syncthreads();
    if (tid < D) {
        float mx = -INFINITY;
#pragma unroll
        for (int g2 = 0; g2 < NG; ++g2) mx = fmaxf(mx, s_acc[g2][D + 2]);
        float a = 0.f, ls = 0.f, cs = 0.f;
#pragma unroll
        for (int g2 = 0; g2 < NG; ++g2) {
            const float mg = s_acc[g2][D + 2];
            const float wgt = (mg == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(mg - mx);
            a = fmaf(wgt, s_acc[g2][tid], a);
            ls = fmaf(wgt, s_acc[g2][D], ls);
            cs += s_acc[g2][D + 1];
        }
        out[(size_t)bhq * D + tid] = dec_from_f32<T>(ls > 0.f ? a / ls : 0.f);
        if (tid == 0) {
            if (lse) lse[bhq] = (mx + __builtin_amdgcn_logf(ls)) * (1.f / DEC_LOG2E);
            if (row_pairs) row_pairs[bhq] = (int32_t)(cs + 0.5f);
        }
    }
}

}  // namespace

hipError_t launch_decode_prefill(const DecodeLayout& L, int n_ctx, const void* kc, const float* cents,
                                 const uint32_t* token_masks, char* st, hipStream_t s)
{
    // counts start at zero even when nothing is cached yet (a fill kernel, not a memset: callers may capture this)
    const int ncount = (int)((L.off_wp - L.off_counts) / 4) + L.B * L.Hkv * L.K;      // counts, padding, window pointers
    hipLaunchKernelGGL(decode_zero_kernel, dim3((ncount + 255) / 256), dim3(256), 0, s, (int*)(st + L.off_counts), ncount);
    if (n_ctx == 0) return hipGetLastError();
    dim3 g1((n_ctx + 255) / 256, L.B * L.Hkv);
    if (token_masks) {
        hipLaunchKernelGGL(decode_prefill_masks_kernel, g1, dim3(256), 0, s, L, n_ctx, token_masks, st);
        hipLaunchKernelGGL(decode_prefill_lists_kernel, dim3(L.K, L.B * L.Hkv), dim3(256), 0, s, L, n_ctx, st);
        return hipGetLastError();
    }
#define FOCUS_DEC_SCORE(T_, KM_) hipLaunchKernelGGL((decode_prefill_score_kernel<T_, KM_>), g1, dim3(256), 0, s, L, n_ctx, (const T_*)kc, cents, st)
    if (L.dtype == 0) {
        if (L.K <= 4) FOCUS_DEC_SCORE(float, 4); else if (L.K <= 8) FOCUS_DEC_SCORE(float, 8);
        else if (L.K <= 16) FOCUS_DEC_SCORE(float, 16); else FOCUS_DEC_SCORE(float, 32);
    } else if (L.dtype == 2) {
        if (L.K <= 4) FOCUS_DEC_SCORE(f16_bits, 4); else if (L.K <= 8) FOCUS_DEC_SCORE(f16_bits, 8);
        else if (L.K <= 16) FOCUS_DEC_SCORE(f16_bits, 16); else FOCUS_DEC_SCORE(f16_bits, 32);
    } else {
        if (L.K <= 4) FOCUS_DEC_SCORE(uint16_t, 4); else if (L.K <= 8) FOCUS_DEC_SCORE(uint16_t, 8);
        else if (L.K <= 16) FOCUS_DEC_SCORE(uint16_t, 16); else FOCUS_DEC_SCORE(uint16_t, 32);
    }
#undef FOCUS_DEC_SCORE
    hipLaunchKernelGGL(decode_prefill_lists_kernel, dim3(L.K, L.B * L.Hkv), dim3(256), 0, s, L, n_ctx, st);
    return hipGetLastError();
}

template <typename T, int D>
static hipError_t decode_step_d(const DecodeLayout& L, const HeadMap& hm, int pos, const int* pos_dev, const T* q_new, const T* kc, const T* vc,
                                char* st, T* out, float* lse, int32_t* row_pairs, hipStream_t s)
{
    float* part = (float*)(st + L.off_part);
    // grouped-query form when query heads hk*G .. hk*G+G-1 share KV head hk (the default map)
    const int G = (L.Hq % L.Hkv == 0) ? L.Hq / L.Hkv : 0;
    bool default_map = G >= 1;
    for (int h = 0; default_map && h < L.Hq; ++h) default_map = hm.kv[h] == h / G;
    // the vector form is built for 1, 2, 4 and 8 heads per KV head; the matrix-core form takes any number (more
    // than 16 in sub-groups of 16, each walking the keys of its own heads)
    bool grouped = default_map && (G == 1 || G == 2 || G == 4 || G == 8);
    // upper bound of the key sequence known on the host: pos + 1 entries.  The lists are walked only while they
    // hold fewer entries than there are positions below the window, the positions themselves otherwise.
    // (With the position in device memory: the bound of the last position the caches can hold; work-groups
    // past the real sequence leave an empty partial.)
    if (pos_dev) pos = L.n - 1;
    int nchunks = std::min(L.max_chunks, (pos + DEC_CHUNK) / DEC_CHUNK);
    // a work-group walks `span` chunks and leaves one partial: at most DEC_MAX_PARTS partials per head, so the
    // merge stays short at any context length
    int span = (nchunks + DEC_MAX_PARTS - 1) / DEC_MAX_PARTS;
    int nparts = (nchunks + span - 1) / span;
    if (sizeof(T) == 2 && default_map && (size_t)L.n * D * 2 <= 0xffffffffull) grouped = true;
    if (grouped) {
        dim3 grid(nparts, L.B * L.Hkv);
        // 16-bit caches whose byte offsets fit 32 bits: the matrix-core form
        if constexpr (sizeof(T) == 2) {
            if ((size_t)L.n * D * 2 <= 0xffffffffull) {
                grid.y = L.B * L.Hkv * ((G + 15) / 16);
                // shorter chunks (fewer rounds per wavefront) while all their work-groups are resident at once, three
                // per CU: below that the long chunks leave most of the chip idle (4096 cached tokens: 27 -> 20 us)
                int ch = DEC_CHUNK;
                for (int c = DEC_CHUNK_SHORT; c < DEC_CHUNK; c *= 2) {
                    const int nc = (pos + c) / c;
                    if ((long)nc * grid.y <= 3 * 256 && nc <= L.max_parts) { ch = c; break; }
                }
                if (ch != DEC_CHUNK) {
                    nchunks = (pos + ch) / ch;
                    span = 1;                                                // one chunk, one partial per work-group
                    nparts = nchunks;
                    grid.x = nparts;
                }
                constexpr bool f16 = std::is_same<T, f16_bits>::value;
#define FOCUS_DEC_MFMA(CH_) hipLaunchKernelGGL((decode_attn_gqa_mfma_kernel<f16, D, CH_>), grid, dim3(256), 0, s, L, G, pos, pos_dev, span, \
                                               (const uint16_t*)q_new, (const uint16_t*)kc, (const uint16_t*)vc, (const char*)st, part)
                if (ch == DEC_CHUNK_SHORT) FOCUS_DEC_MFMA(DEC_CHUNK_SHORT);
                else if (ch == 2 * DEC_CHUNK_SHORT) FOCUS_DEC_MFMA(2 * DEC_CHUNK_SHORT);
                else FOCUS_DEC_MFMA(DEC_CHUNK);
#undef FOCUS_DEC_MFMA
                hipLaunchKernelGGL((decode_merge_kernel<T, D>), dim3(L.B * L.Hq), dim3(256), 0, s, L, pos, pos_dev, nparts, part, out,
                                   lse, row_pairs);
                return hipGetLastError();
            }
        }
#define FOCUS_DEC_GQA(G_) hipLaunchKernelGGL((decode_attn_gqa_kernel<T, D, G_>), grid, dim3(256), 0, s, L, pos, pos_dev, span, q_new, kc, vc, (const char*)st, part)
        if (G == 1) FOCUS_DEC_GQA(1); else if (G == 2) FOCUS_DEC_GQA(2); else if (G == 4) FOCUS_DEC_GQA(4); else FOCUS_DEC_GQA(8);
#undef FOCUS_DEC_GQA
    } else {
        hipLaunchKernelGGL((decode_attn_kernel<T, D>), dim3(nparts, L.B * L.Hq), dim3(256), 0, s, L, hm, pos, pos_dev, span,
                           q_new, kc, vc, (const char*)st, part);
    }
    hipLaunchKernelGGL((decode_merge_kernel<T, D>), dim3(L.B * L.Hq), dim3(256), 0, s, L, pos, pos_dev, nparts, part, out, lse,
                       row_pairs);
    return hipGetLastError();
}

template <typename T>
static hipError_t decode_step_t(const DecodeLayout& L, const HeadMap& hm, int pos, const int* pos_dev, const void* q_new, const void* k_new,
                                const void* v_new, const float* cents, const uint32_t* token_mask, void* kc, void* vc, char* st, void* out,
                                float* lse, int32_t* row_pairs, hipStream_t s)
{
    hipLaunchKernelGGL(decode_route_kernel<T>, dim3(L.Hq + L.Hkv, L.B), dim3(64), 0, s, L, hm, pos, pos_dev, (const T*)q_new,
                       (const T*)k_new, (const T*)v_new, cents, token_mask, (T*)kc, (T*)vc, st);
#define FOCUS_DEC_D(D_) decode_step_d<T, D_>(L, hm, pos, pos_dev, (const T*)q_new, (const T*)kc, (const T*)vc, st, (T*)out, lse, row_pairs, s)
    switch (L.d) {
        case 64: return FOCUS_DEC_D(64);
        case 80: return FOCUS_DEC_D(80);
        case 96: return FOCUS_DEC_D(96);
        case 128: return FOCUS_DEC_D(128);
        case 256: return FOCUS_DEC_D(256);
        default: return hipErrorInvalidValue;
    }
#undef FOCUS_DEC_D
}

hipError_t launch_decode_step(const DecodeLayout& L, const HeadMap& hm, int pos, const int* pos_dev, const void* q_new, const void* k_new,
                              const void* v_new, const float* cents, const uint32_t* token_mask, void* kc, void* vc, char* st, void* out, float* lse,
                              int32_t* row_pairs, hipStream_t s)
{
    if (L.dtype == 0)
        return decode_step_t<float>(L, hm, pos, pos_dev, q_new, k_new, v_new, cents, token_mask, kc, vc, st, out, lse, row_pairs, s);
    if (L.dtype == 2)
        return decode_step_t<f16_bits>(L, hm, pos, pos_dev, q_new, k_new, v_new, cents, token_mask, kc, vc, st, out, lse, row_pairs, s);
    return decode_step_t<uint16_t>(L, hm, pos, pos_dev, q_new, k_new, v_new, cents, token_mask, kc, vc, st, out, lse, row_pairs, s);
}

}  // namespace focus
