// Block-sparse flash-style attention forward on the gfx950 matrix cores
// (bf16 in, fp32 accumulate): App. D Eq. 3 generalised to top-k sets, exact
// softmax (Sec. 1), every allowed pair visited once under ONE online softmax.
//
// Data layout (built by the two gather kernels below, class order = tokens
// bucketed by membership class, position-ascending inside a class, every class
// segment padded to a multiple of KT with position KPOS_PAD and zero data):
//   Kc [B*Hkv][NKP][D]            keys, row-major: a key tile is one contiguous block
//   Vt [B*Hkv][NKP/KT][D][KT]     values, transposed per key tile (KT = 64 keys), the 16 keys of
//                                 every 16-key group stored in MFMA k-slot order
// One work-group = 4 wavefronts = one query tile of BQ=128 rows of one class;
// each wavefront owns 32 query rows.  The scores are computed transposed,
// S^T = K Q^T with v_mfma_f32_32x32x16_bf16 (A = K rows from LDS, B = Q rows held
// in registers), so that one lane holds 16x4 scores of ONE query row: row max
// and row sum are in-lane reductions plus one exchange between the two half
// waves.  The probabilities, rounded to bf16, are already laid out as the B
// operand of O^T += V^T P^T; the A operand comes from the transposed V tile.
#include "focus_internal.h"
#include "focus_tileplan.h"
#include <cstdlib>

namespace focus {

namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));   // native 16-byte vector (keeps staging in registers)

constexpr int NTHR = 256;
constexpr float LOG2E = 1.4426950408889634f;

// within a 16-key group: MFMA k-slot p16 = h*8 + e  <->  key 8*(e/4) + 4*h + e%4,
// the order in which a lane of the S^T accumulator holds its keys
__host__ __device__ constexpr int slot_to_key16(int p16) { return 8 * ((p16 % 8) / 4) + 4 * (p16 / 8) + (p16 % 8) % 4; }

// ---------------------------------------------------------------- gathers into class order
template <int D>
__global__ __launch_bounds__(NTHR) void gather_k_kernel(Layout L, const uint16_t* __restrict__ k, char* __restrict__ ws)
{
    constexpr int CPR = D / 8;                       // 16-byte chunks per row
    const int tile = blockIdx.x, bhk = blockIdx.y, tid = threadIdx.x;
    const int* kpos = (const int*)(ws + L.off_kpos) + (size_t)bhk * L.NKP + (size_t)tile * KT;
    uint4* dst = (uint4*)(ws + L.off_kc) + ((size_t)bhk * L.NKP + (size_t)tile * KT) * CPR;
    const uint4* src = (const uint4*)k + (size_t)bhk * L.n * CPR;
    for (int id = tid; id < KT * CPR; id += NTHR) {
        const int row = id / CPR, ch = id % CPR;
        const int kp = kpos[row];
        uint4 val = make_uint4(0, 0, 0, 0);
        if (kp != KPOS_PAD) val = src[(size_t)kp * CPR + ch];
        dst[id] = val;
    }
}

template <int D>
__global__ __launch_bounds__(NTHR) void gather_vt_kernel(Layout L, const uint16_t* __restrict__ v, char* __restrict__ ws)
{
    constexpr int CPR = D / 8;
    constexpr int RS = D + 2;                        // padded LDS row stride in elements
    __shared__ uint16_t s_v[KT * RS];
    const int tile = blockIdx.x, bhk = blockIdx.y, tid = threadIdx.x;
    const int* kpos = (const int*)(ws + L.off_kpos) + (size_t)bhk * L.NKP + (size_t)tile * KT;
    const uint4* src = (const uint4*)v + (size_t)bhk * L.n * CPR;
    for (int id = tid; id < KT * CPR; id += NTHR) {
        const int row = id / CPR, ch = id % CPR;
        const int kp = kpos[row];
        uint4 val = make_uint4(0, 0, 0, 0);
        if (kp != KPOS_PAD) val = src[(size_t)kp * CPR + ch];
        uint32_t* d32 = (uint32_t*)(s_v + row * RS + ch * 8);   // RS even -> 4-byte aligned
        d32[0] = val.x; d32[1] = val.y; d32[2] = val.z; d32[3] = val.w;
    }
    __syncthreads();
    uint4* dst = (uint4*)(ws + L.off_vt) + ((size_t)bhk * (L.NKP / KT) + tile) * (size_t)(D * KT / 8);
    for (int id = tid; id < D * (KT / 8); id += NTHR) {
        const int drow = id / (KT / 8), c = id % (KT / 8);
        uint16_t e[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int p = c * 8 + j;
            const int key = (p / 16) * 16 + slot_to_key16(p % 16);
            e[j] = s_v[key * RS + drow];
        }
        uint4 val;
        val.x = e[0] | ((uint32_t)e[1] << 16); val.y = e[2] | ((uint32_t)e[3] << 16);
        val.z = e[4] | ((uint32_t)e[5] << 16); val.w = e[6] | ((uint32_t)e[7] << 16);
        dst[id] = val;
    }
}

// ---------------------------------------------------------------- attention
// 16-byte chunk swizzle: 16 consecutive rows must land on 16 different chunk slots of a
// 256-byte bank line.  Rows of 256 bytes: slot ^= row & 15; rows of 128 bytes: slot ^= (row >> 1) & 7.
template <int ROW_BYTES>
__device__ inline int swz(int row, int ch)
{
    if constexpr (ROW_BYTES == 256) return ch ^ (row & 15);
    else return ch ^ ((row >> 1) & 7);
}

template <int D>
struct Smem {
    TilePlan plan;
    int kpos[KT];
    __attribute__((aligned(16))) char k[KT * D * 2];     // [key][D] bf16, chunks swizzled
    __attribute__((aligned(16))) char vt[D * KT * 2];    // [d][KT] bf16, chunks swizzled
};

template <int D, bool SOFTCAP, bool PAIRS>
__global__ __launch_bounds__(NTHR, 2) void attn_mfma_kernel(Layout L, HeadMap hm, int default_map,
                                                            const uint16_t* __restrict__ q,
                                                            const char* __restrict__ ws, uint16_t* __restrict__ out,
                                                            float* __restrict__ lse, int32_t* __restrict__ row_pairs)
{
    __shared__ Smem<D> S;
    constexpr int KS = D / 16;          // k-steps of the QK^T contraction
    constexpr int DB = D / 32;          // 32-row blocks of O^T
    constexpr int KCH = D / 8;          // 16-byte chunks per key row
    constexpr int KB = KT / 32;         // 32-key blocks per tile
    constexpr int NLK = KT * KCH / NTHR;        // 16-byte loads per thread for a K tile
    constexpr int NLV = D * (KT / 8) / NTHR;    // ... and for a V^T tile
    constexpr int VCH = KT / 8;                 // chunks per V^T row
    constexpr float RESCALE_THRESHOLD = 8.f;    // log2 units the row max may drift before O is rescaled

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n32 = lane & 31, hh = lane >> 5;

    // work-group -> (job slot, head): heads fastest so the heavy slots of all heads start
    // first; with the default head map the query heads of one KV head share blockIdx % 8
    const int BH = L.B * L.Hq;
    const int job = blockIdx.x / BH;
    const int x = blockIdx.x % BH;
    int b, h;
    if (default_map) {
        const int BHk = L.B * L.Hkv, G = L.Hq / L.Hkv;
        const int kvlin = x % BHk, g = x / BHk;
        b = kvlin / L.Hkv;
        h = (kvlin % L.Hkv) * G + g;
    } else {
        b = x / L.Hq;
        h = x % L.Hq;
    }
    const int bhq = b * L.Hq + h;
    const int bhk = b * L.Hkv + hm.kv[h];
    if (!plan_query_tile(L, ws, bhq, bhk, job, S.plan)) return;

    const int rloc = wave * 32 + n32;                       // query row inside the tile
    const bool rvalid = rloc < S.plan.nvalid;
    const int* qperm = (const int*)(ws + L.off_qperm) + (size_t)bhq * L.NQP;
    const int qpos = rvalid ? qperm[S.plan.row0 + rloc] : -1;
    const int i_lo = S.plan.i_lo;
    const int total = S.plan.total;
    const int w = L.window;

    // Q rows as the B operand: lane (n32, hh) holds Q[row][16*ks + 8*hh .. +7]
    bf16x8 qreg[KS];
    {
        const bf16x8* qrow = (const bf16x8*)(q + ((size_t)bhq * L.n + (rvalid ? qpos : 0)) * D);
        bf16x8 zero;
#pragma unroll
        for (int e = 0; e < 8; ++e) zero[e] = (__bf16)0.f;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) qreg[ks] = rvalid ? qrow[2 * ks + hh] : zero;
    }

    f32x16 o[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[db][r] = 0.f;
    float m_ref = -INFINITY;   // reference max of the row in log2 units (may lag the true max)
    float l_run = 0.f;         // this lane's share of the running sum
    int npairs = 0;

    const float sl2 = L.scale * LOG2E;
    const float cap_l2 = L.softcap * LOG2E;
    const float two_over_cap_l2 = (L.softcap > 0.f) ? 2.f * L.scale * LOG2E / L.softcap : 0.f;

    const u32x4* kc_base = (const u32x4*)(ws + L.off_kc) + (size_t)bhk * L.NKP * KCH;
    const u32x4* vt_base = (const u32x4*)(ws + L.off_vt) + (size_t)bhk * L.NKP * KCH;
    const int* kpos_base = (const int*)(ws + L.off_kpos) + (size_t)bhk * L.NKP;

    // register staging of the next tile: global loads fly while the current tile is computed
    u32x4 st_k[NLK], st_v[NLV];
    int st_kpos;
#define FOCUS_ISSUE_LOADS(TILE)                                                              \
    do {                                                                                     \
        const u32x4* ksrc_ = kc_base + (size_t)(TILE) * (KT * KCH);                          \
        _Pragma("unroll") for (int i = 0; i < NLK; ++i) st_k[i] = ksrc_[tid + i * NTHR];     \
        const u32x4* vsrc_ = vt_base + (size_t)(TILE) * (D * VCH);                           \
        _Pragma("unroll") for (int i = 0; i < NLV; ++i) st_v[i] = vsrc_[tid + i * NTHR];     \
        st_kpos = kpos_base[(size_t)(TILE) * KT + (tid & (KT - 1))];                         \
    } while (0)
#define FOCUS_COMMIT_LOADS()                                                                 \
    do {                                                                                     \
        _Pragma("unroll") for (int i = 0; i < NLK; ++i) {                                    \
            const int id_ = tid + i * NTHR;                                                  \
            const int row_ = id_ / KCH, ch_ = id_ % KCH;                                     \
            *(u32x4*)(S.k + row_ * (D * 2) + swz<D * 2>(row_, ch_) * 16) = st_k[i];          \
        }                                                                                    \
        _Pragma("unroll") for (int i = 0; i < NLV; ++i) {                                    \
            const int id_ = tid + i * NTHR;                                                  \
            const int row_ = id_ / VCH, ch_ = id_ % VCH;                                     \
            *(u32x4*)(S.vt + row_ * (KT * 2) + swz<KT * 2>(row_, ch_) * 16) = st_v[i];       \
        }                                                                                    \
        if (tid < KT) S.kpos[tid] = st_kpos;                                                 \
    } while (0)

    if (total == 0) return;      // cannot happen (the diagonal is always allowed); keeps the loads in bounds
    int cur = 0, cur_ld = 0;
    int tile_ld = S.plan.t0[0];
    while (0 >= S.plan.cum[cur_ld + 1]) ++cur_ld;
    tile_ld = S.plan.t0[cur_ld];
    FOCUS_ISSUE_LOADS(tile_ld);
    FOCUS_COMMIT_LOADS();
    for (int it = 0; it < total; ++it) {
        while (it >= S.plan.cum[cur + 1]) ++cur;
        const bool inter = S.plan.inter[cur] != 0;
        __syncthreads();                                     // tile `it` is in LDS
        if (it + 1 < total) {                                // next tile (the last one is re-read, harmlessly)
            while (it + 1 >= S.plan.cum[cur_ld + 1]) ++cur_ld;
            tile_ld = S.plan.t0[cur_ld] + (it + 1 - S.plan.cum[cur_ld]);
        }
        FOCUS_ISSUE_LOADS(tile_ld);

        // ---- S^T = K Q^T: KB blocks of 32 keys x 32 queries per wavefront
        f32x16 s[KB];
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) {
#pragma unroll
            for (int r = 0; r < 16; ++r) s[kb][r] = 0.f;
            const int row = kb * 32 + n32;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                bf16x8 a = *(const bf16x8*)(S.k + row * (D * 2) + swz<D * 2>(row, 2 * ks + hh) * 16);
                s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qreg[ks], s[kb], 0, 0, 0);
            }
        }

        // ---- softcap (to log2 units) and mask
        if constexpr (SOFTCAP) {
#pragma unroll
            for (int kb = 0; kb < KB; ++kb)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    // cap*tanh(scale*x/cap) = cap*(1 - 2/(1+exp(2*scale*x/cap))), in log2 units
                    const float e2 = __builtin_amdgcn_exp2f(s[kb][r] * two_over_cap_l2);
                    s[kb][r] = cap_l2 - 2.f * cap_l2 * __builtin_amdgcn_rcpf(1.f + e2);
                }
        }
        const bool interior = inter && (S.kpos[KT - 1] <= i_lo);
        if (!interior) {
#pragma unroll
            for (int kb = 0; kb < KB; ++kb) {
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    const int4 kp4 = *(const int4*)(&S.kpos[kb * 32 + 8 * r4 + 4 * hh]);
                    const int kp[4] = {kp4.x, kp4.y, kp4.z, kp4.w};
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const bool ok = kp[e] <= qpos && (inter || kp[e] > qpos - w);
                        s[kb][r4 * 4 + e] = ok ? s[kb][r4 * 4 + e] : -INFINITY;
                        if constexpr (PAIRS) npairs += ok ? 1 : 0;
                    }
                }
            }
        } else {
            if constexpr (PAIRS) npairs += KT / 2;
        }

        // ---- online softmax (one row per lane pair); the reference max is only moved when
        //      the true max has drifted by more than the threshold, so O is rarely rescaled
        float mx = -INFINITY;
#pragma unroll
        for (int kb = 0; kb < KB; ++kb)
#pragma unroll
            for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[kb][r]);
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        const float m2 = SOFTCAP ? mx : mx * sl2;            // scale > 0: max commutes with scaling
        const bool upd = m2 > m_ref + RESCALE_THRESHOLD;     // m_ref = -inf: any finite max updates
        if (__any(upd)) {
            const float alpha = upd ? __builtin_amdgcn_exp2f(m_ref - m2) : 1.f;
            m_ref = upd ? m2 : m_ref;
            l_run *= alpha;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int r = 0; r < 16; ++r) o[db][r] *= alpha;
        }
        const float m_use = (m_ref == -INFINITY) ? 0.f : m_ref;
        float psum = 0.f;
        bf16x8 pb[KB][2];
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float arg = SOFTCAP ? (s[kb][r] - m_use) : fmaf(s[kb][r], sl2, -m_use);
                const float p = __builtin_amdgcn_exp2f(arg);
                psum += p;
                pb[kb][r / 8][r % 8] = (__bf16)p;
            }
        }
        l_run += psum;

        // ---- O^T += V^T P^T
#pragma unroll
        for (int db = 0; db < DB; ++db) {
            const int row = db * 32 + n32;
#pragma unroll
            for (int kb = 0; kb < KB; ++kb) {
#pragma unroll
                for (int s2 = 0; s2 < 2; ++s2) {
                    bf16x8 a = *(const bf16x8*)(S.vt + row * (KT * 2) + swz<KT * 2>(row, kb * 4 + s2 * 2 + hh) * 16);
                    o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pb[kb][s2], o[db], 0, 0, 0);
                }
            }
        }
        __syncthreads();                                     // every wavefront is done with tile `it`
        FOCUS_COMMIT_LOADS();
    }
#undef FOCUS_ISSUE_LOADS
#undef FOCUS_COMMIT_LOADS

    // ---- epilogue
    const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
    if constexpr (PAIRS) npairs += __shfl_xor(npairs, 32, 64);
    if (!rvalid) return;
    const float inv = 1.f / l_tot;
    uint16_t* orow = out + ((size_t)bhq * L.n + qpos) * D;
#pragma unroll
    for (int db = 0; db < DB; ++db) {
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
            const int dcol = db * 32 + 8 * r4 + 4 * hh;
            __bf16 e0 = (__bf16)(o[db][r4 * 4 + 0] * inv), e1 = (__bf16)(o[db][r4 * 4 + 1] * inv);
            __bf16 e2 = (__bf16)(o[db][r4 * 4 + 2] * inv), e3 = (__bf16)(o[db][r4 * 4 + 3] * inv);
            uint16_t u0, u1, u2, u3;
            __builtin_memcpy(&u0, &e0, 2); __builtin_memcpy(&u1, &e1, 2);
            __builtin_memcpy(&u2, &e2, 2); __builtin_memcpy(&u3, &e3, 2);
            uint2 val;
            val.x = u0 | ((uint32_t)u1 << 16);
            val.y = u2 | ((uint32_t)u3 << 16);
            *(uint2*)(orow + dcol) = val;
        }
    }
    if (hh == 0) {
        if (lse) lse[(size_t)bhq * L.n + qpos] = (m_ref + __builtin_amdgcn_logf(l_tot)) * (1.f / LOG2E);
        if constexpr (PAIRS) row_pairs[(size_t)bhq * L.n + qpos] = npairs;
    }
}

template <int D, bool SOFTCAP, bool PAIRS>
hipError_t launch_one(const Layout& L, const HeadMap& hm, int default_map, const void* q, char* ws, void* out,
                      float* lse, int32_t* row_pairs, hipStream_t st)
{
    auto kern = attn_mfma_kernel<D, SOFTCAP, PAIRS>;
    const unsigned grid = (unsigned)((size_t)L.NT * L.B * L.Hq);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(NTHR), 0, st, L, hm, default_map, (const uint16_t*)q,
                       (const char*)ws, (uint16_t*)out, lse, row_pairs);
    return hipGetLastError();
}

template <int D>
hipError_t launch_d(const Layout& L, const HeadMap& hm, int default_map, const void* q, const void* v, char* ws,
                    void* out, float* lse, int32_t* row_pairs, hipStream_t st)
{
    dim3 ggrid(L.NKP / KT, L.B * L.Hkv);
    hipLaunchKernelGGL(gather_vt_kernel<D>, ggrid, dim3(NTHR), 0, st, L, (const uint16_t*)v, ws);
    const bool sc = L.softcap > 0.f, pairs = row_pairs != nullptr;
    static const int variant = [] { const char* e = getenv("FOCUS_MFMA_VARIANT"); return e ? atoi(e) : 3; }();
    if (variant == 3) return launch_attn_mfma3_core(L, hm, default_map, q, ws, out, lse, row_pairs, st);
    if (sc) {
        return pairs ? launch_one<D, true, true>(L, hm, default_map, q, ws, out, lse, row_pairs, st)
                     : launch_one<D, true, false>(L, hm, default_map, q, ws, out, lse, row_pairs, st);
    }
    return pairs ? launch_one<D, false, true>(L, hm, default_map, q, ws, out, lse, row_pairs, st)
                 : launch_one<D, false, false>(L, hm, default_map, q, ws, out, lse, row_pairs, st);
}

}  // namespace

// Class-ordered copy of the keys; part of focus_assign for bf16 problems.
hipError_t launch_gather_k(const Layout& L, const void* k, char* ws, hipStream_t st)
{
    dim3 ggrid(L.NKP / KT, L.B * L.Hkv);
    if (L.d == 64)
        hipLaunchKernelGGL(gather_k_kernel<64>, ggrid, dim3(NTHR), 0, st, L, (const uint16_t*)k, ws);
    else
        hipLaunchKernelGGL(gather_k_kernel<128>, ggrid, dim3(NTHR), 0, st, L, (const uint16_t*)k, ws);
    return hipGetLastError();
}

hipError_t launch_attn_mfma(const Layout& L, const HeadMap& hm, const void* q, const void* k, const void* v,
                            char* ws, void* out, float* lse, int32_t* row_pairs, hipStream_t st)
{
    (void)k;
    int default_map = 1;
    const int G = L.Hq / L.Hkv;
    if (L.Hq % L.Hkv != 0) default_map = 0;
    else
        for (int h = 0; h < L.Hq; ++h)
            if (hm.kv[h] != h / G) default_map = 0;
    if ((size_t)L.NT * L.B * L.Hq > 0x7fffffffull) return hipErrorInvalidValue;
    if (L.d == 64) return launch_d<64>(L, hm, default_map, q, v, ws, out, lse, row_pairs, st);
    return launch_d<128>(L, hm, default_map, q, v, ws, out, lse, row_pairs, st);
}

}  // namespace focus
