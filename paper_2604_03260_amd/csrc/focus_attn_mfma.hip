// Block-sparse flash-style attention forward on the gfx950 matrix cores
// (bf16 or fp16 in, fp32 accumulate): App. D Eq. 3 generalised to top-k sets, exact
// softmax (Sec. 1), every allowed pair visited once under ONE online softmax.
//
// Data layout (built by the two gather kernels below, class order = tokens
// bucketed by membership class, position-ascending inside a class, every class
// segment padded to a multiple of KT with position KPOS_PAD and zero data):
//   Kc [B*Hkv][NKP][D]            keys, row-major: a key tile is one contiguous block
//   Vt [B*Hkv][NKP/KT][D][KT]     values, transposed per key tile (KT = 64 keys), the 16 keys of
//                                 every 16-key group stored in MFMA k-slot order
// D is the head dim rounded up to 64, 128 or 256 (zero columns / rows past it); the kernel runs
// KS = d/16 k-steps of Q K^T and DB = ceil(d/32) row blocks of O^T, so a head dim of 80 or 96
// pays for its own products only.
// One work-group = MFMA_WAVES wavefronts = one query tile of 32*MFMA_WAVES rows of one class;
// each wavefront owns 32 query rows.  The scores are computed transposed,
// S^T = K Q^T with v_mfma_f32_32x32x16_bf16 (A = K rows from LDS, B = Q rows held
// in registers), so that one lane holds 16 scores of ONE query row per 32-key
// unit: row max and row sum are in-lane reductions plus one exchange between
// the two half waves.  The probabilities, rounded to bf16, are already laid out
// as the B operand of O^T += V^T P^T; the A operand comes from the transposed V tile.
//
// How a wavefront's work is ordered and how tiles reach LDS:
//  * A key tile of 64 is two units of 32 keys.  While the vector ALUs turn the
//    scores of one unit into probabilities, the matrix cores run the products of
//    its neighbours, inside ONE instruction stream:
//      phase A of tile t:  MFMA  O += V(t-1,u1) P1(t-1)   and   S1 = K(t,u1) Q^T
//                          VALU  P0 = softmax-step(S0)
//      phase B of tile t:  MFMA  O += V(t,u0) P0          and   S0 = K(t+1,u0) Q^T
//                          VALU  P1 = softmax-step(S1)
//    The 16 LDS operands of a phase are read as one batch at its start.
//  * K and V^T tiles are double-buffered in LDS and filled with
//    global_load_lds_dwordx4: 64 lanes x 16 bytes land at M0 + lane*16.  LDS rows
//    are 16 bytes longer than their data (bank-conflict-free operand reads whose
//    chunk is an immediate offset), so each lane fetches the global chunk that
//    belongs in its LDS slot.  The loads of K(t+2), V(t+1) and the key positions
//    of tile t+2 are issued in the middle of tile t, right after the one barrier
//    per tile, and waited for with s_waitcnt vmcnt(0) just before the next one.
//  * Softmax without a reference where the data allow it.  softmax is invariant under a shift of the logits,
//    so the usual running row max is only there to keep exp in range.  focus_assign leaves the largest squared
//    key norm of every KV head in the workspace; with |q_i| from the row itself, Cauchy-Schwarz bounds every
//    logit of row i (log2 units) by b_i = scale*log2(e)*|q_i|*max|k| (and by the cap, with a softcap).  A
//    work-group whose rows all have b_i <= NOREF_BOUND takes p = exp2(logit) as it is, in [2^-60, 2^60]: no row
//    max, no exchange between the half-waves, no rescaling of O, and (without a softcap) no multiply-subtract
//    either, because the query rows are pre-multiplied by scale*log2(e) when they are loaded (one more 16-bit
//    rounding of q, a relative 2^-9 per component: about 1e-3 absolute in a logit, below the rounding of the
//    16-bit probabilities).  The sums stay far inside fp32 (2^60 * 2^24 keys * |v|), and out = O / l is the same
//    exact softmax.  Any other work-group (large norms, non-finite keys) runs the second copy of the loop:
//  * there the reference max of a row only moves when the true max has drifted
//    by more than RESCALE_THRESHOLD (log2 units), so O is rarely rescaled.
//  * The row sum adds the bf16-rounded probabilities (v_dot2), the numbers PV uses.
#include "focus_internal.h"
#include "focus_tileplan.h"
#include <algorithm>
#include <type_traits>

namespace focus {

namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
typedef __attribute__((__vector_size__(8 * sizeof(_Float16)))) _Float16 f16x8;
typedef __attribute__((__vector_size__(2 * sizeof(_Float16)))) _Float16 f16x2;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

// the two 16-bit element types: vector types, the 32x32x16 product and the 2-term dot product
template <bool F16> struct Half;
template <> struct Half<false> {
    typedef __bf16 T;
    typedef bf16x8 V8;
    typedef bf16x2 V2;
    static __device__ inline f32x16 mfma(V8 a, V8 b, f32x16 c) { return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0); }
    static __device__ inline float dot2(V2 a, V2 b, float c) { return __builtin_amdgcn_fdot2_f32_bf16(a, b, c, false); }
};
template <> struct Half<true> {
    typedef _Float16 T;
    typedef f16x8 V8;
    typedef f16x2 V2;
    static __device__ inline f32x16 mfma(V8 a, V8 b, f32x16 c) { return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0); }
    static __device__ inline float dot2(V2 a, V2 b, float c) { return __builtin_amdgcn_fdot2(a, b, c, false); }
};
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int NTHR = 256;

// Timing-only builds for the loop ablation under profiles/ (python build.py --ablate BITS; never in libfocus.so).
// Each bit takes one ingredient out of the key-tile loop so that its share of the time can be read off; the
// results of such a build are meaningless.  Every variant stays inside its buffers and waits for nothing that
// does not come: 1 = no barrier per tile (wavefronts may read a stage another one is still filling),
// 2 = no v_exp_f32 (the probabilities are the converted logits), 4 = no K/V tile DMA in the loop (every tile
// re-reads what the prologue loaded), 8 = no LDS operand reads in the loop (the MFMAs run on the registers'
// last contents), 16 = no wait for the tile DMA inside the loop (a tile may be read before it has landed; the wait
// after the loop stays).
#ifndef FOCUS_ABLATE
#define FOCUS_ABLATE 0
#endif
constexpr float LOG2E = 1.4426950408889634f;
constexpr float RESCALE_THRESHOLD = 8.f;    // log2 units the row max may drift before O is rescaled
constexpr float NOREF_BOUND = 60.f;         // largest |logit| bound (log2 units) up to which exp2 needs no reference
constexpr float NOREF_SLACK = 1.01f;        // the bound is taken this much larger than computed (fp32 rounding of the norms)
constexpr float CAP_POLY_Z = 0.3f;          // |score*scale/softcap| up to which tanh is taken as its Taylor polynomial to z^5
constexpr float CAP_CUBIC_Z = 0.15f;        // ... and to z^3 (the z^5 term is then below 7.3e-4 log2 units at cap 50)

// within a 16-key group: MFMA k-slot p16 = h*8 + e  <->  key 8*(e/4) + 4*h + e%4,
// the order in which a lane of the S^T accumulator holds its keys
__host__ __device__ constexpr int slot_to_key16(int p16) { return 8 * ((p16 % 8) / 4) + 4 * (p16 / 8) + (p16 % 8) % 4; }

// ---------------------------------------------------------------- gathers into class order
template <int D>
__global__ __launch_bounds__(NTHR) void gather_vt_kernel(Layout L, const uint16_t* __restrict__ v, char* __restrict__ ws)
{
    constexpr int CPR = D / 8;
    constexpr int RS = D + 2;                        // padded LDS row stride in elements
    __shared__ uint16_t s_v[KT * RS];
    const int cin = L.d / 8;
    const int tile = blockIdx.x, bhk = blockIdx.y, tid = threadIdx.x;
    const int* kpos = (const int*)(ws + L.off_kpos) + (size_t)bhk * L.NKP + (size_t)tile * KT;
    const uint4* src = (const uint4*)v + ((size_t)(bhk / L.Hkv) * L.ks[0] + (size_t)(bhk % L.Hkv) * L.ks[1]) / 8;
    const size_t pitch = (size_t)L.ks[2] / 8;
    for (int id = tid; id < KT * CPR; id += NTHR) {
        const int row = id / CPR, ch = id % CPR;
        const int kp = kpos[row];
        uint4 val = make_uint4(0, 0, 0, 0);
        if (kp != KPOS_PAD && ch < cin) val = src[(size_t)kp * pitch + ch];
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
constexpr int GROW = 128;     // bytes of a key's soft assignment in LDS: bf16 high parts of 32 groups, then the low parts

// LDS rows of the K and V^T tiles are 16 bytes longer than their data: with pitches of 272 / 528 / 144 bytes
// the 16 lanes of a ds_read_b128 group (16 consecutive rows, the same chunk) fall on 16 different bank
// quads, and the chunk of a read is a compile-time byte offset: every operand read is
// `ds_read_b128 v, vaddr offset:imm` with ONE per-lane address register per operand kind and no address
// arithmetic in the loop.
template <int D> struct TileGeom {
    static constexpr int KROW = D * 2 + 16;             // pitch of a key row
    static constexpr int VROW = KT * 2 + 16;            // pitch of a V^T row (KT keys)
    static constexpr int K_LDS = KT * KROW;             // bytes of a K stage, a multiple of 1024
    static constexpr int V_LDS = D * VROW;              // bytes of a V^T stage, a multiple of 1024
    static_assert(K_LDS % 1024 == 0 && V_LDS % 1024 == 0, "stages are filled in 1-KB wave loads");
};

template <int D, bool COARSE, bool SOFT>
struct Smem {
    TilePlan plan;
    __attribute__((aligned(16))) int kpos[3][KT];
    __attribute__((aligned(16))) char k[2][TileGeom<D>::K_LDS];    // [stage][key][KROW] 16-bit elements
    __attribute__((aligned(16))) char vt[2][TileGeom<D>::V_LDS];   // [stage][d][VROW] 16-bit elements
    __attribute__((aligned(16))) unsigned kmsk[COARSE ? 3 * KT : 4];   // membership masks of the keys (coarse classes)
    __attribute__((aligned(16))) char gk[SOFT ? 2 * KT * GROW : 16];   // [stage][key][GROW] soft assignments of the keys
};

// max of the two half-waves (lane l and lane l^32 hold the same query row)
__device__ inline float halfwave_max(float x)
{
    const unsigned xi = __float_as_uint(x);
    auto r = __builtin_amdgcn_permlane32_swap(xi, xi, false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

// 16-byte LDS read whose completion the compiler does not track (see F4_WAIT_OPERANDS)
template <typename V8>
__device__ inline V8 lds_read16_async(unsigned addr)
{
    V8 r;
    asm volatile("ds_read_b128 %0, %1" : "=v"(r) : "v"(addr));
    return r;
}
// the same with a compile-time byte offset in the instruction
template <typename V8, int OFF>
__device__ inline V8 lds_read16_async_at(unsigned addr)
{
    static_assert(OFF >= 0 && OFF < 65536, "ds offsets are 16 bits");
    V8 r;
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(r) : "v"(addr), "n"(OFF));
    return r;
}
// compile-time loop: f(std::integral_constant<int, I>) for I = 0 .. N-1
template <int I, int N, typename F>
__device__ inline void static_for(F&& f)
{
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, N>(f);
    }
}
// s_waitcnt lgkmcnt(0) tied to every register of an operand array (N = 4..16 registers of 16 bytes)
template <typename V8, int N>
__device__ inline void wait_lds_operands(V8 (&a)[N])
{
    static_assert(N >= 4, "operand arrays hold at least four registers");
    asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(a[0]), "+v"(a[1]), "+v"(a[2]), "+v"(a[3]));
#pragma unroll
    for (int i = 4; i < N; ++i) asm volatile("" : "+v"(a[i]));
}
template <typename V8, int N>
__device__ inline void pin_operands(V8 (&a)[N])
{
#pragma unroll
    for (int i = 0; i < N; ++i) asm volatile("" : "+v"(a[i]));
}

// D: row length of the class-ordered copies (64, 128, 256); KS: MFMAs of one QK^T unit = d / 16;
// DB: 32-row blocks of O^T = ceil(d / 32).  With 512-byte key rows the operands of a phase alone
// take 128 registers, so that shape runs one wavefront per SIMD with the full register file.
// COARSE: membership classes are sets of super-groups; a key class that shares one with the rows' class
// may or may not share a real group, so its pairs are tested against the two membership masks.
// SOFT: Sec. 2 Eq. 2, the attention of training: one class in position order, every causal pair computed; the
// score of a pair outside the window is multiplied by sigmoid(lambda * g_i . g_j).  The affinities come off the
// matrix cores next to the scores: G^T = g_K g_Q^T with both sides split into bf16 high and low parts (three
// products per 16 groups), the query side pre-multiplied by -lambda*log2(e) so that the gate is 1/(1 + 2^G).
// Runs one wavefront per SIMD (two more accumulators and the operands of G do not fit 256 registers).
// NOREF: the softmax without a reference (head of this file).  Every launch runs the kernel twice: the NOREF
// instantiation first, whose work-groups check their bound, leave a flag (1 = done here, 0 = not mine) and do
// the tile or return; then the other instantiation, whose work-groups return at once where the flag says done.
template <int D, int KS, int DB, int MFMA_WAVES, bool SOFTCAP, bool PAIRS, bool F16, bool COARSE, bool SOFT, bool NOREF>
__global__ __launch_bounds__(64 * MFMA_WAVES, (D == 256 || SOFT) ? 1 : 8 / MFMA_WAVES) void attn_mfma_kernel(
    Layout L, HeadMap hm, int default_map, const uint16_t* __restrict__ q, const float* __restrict__ g,
    char* ws_rw, uint16_t* __restrict__ out, float* __restrict__ lse,
    int32_t* __restrict__ row_pairs)
{
    const char* ws = ws_rw;              // everything but the flag of this work-group is only read
    typedef Half<F16> HT;
    typedef typename HT::T elem_t;
    typedef typename HT::V8 V8;
    typedef typename HT::V2 V2;
    __shared__ Smem<D, COARSE, SOFT> S;
    static_assert(KS * 16 <= D && DB * 32 <= D, "the products stay inside the copied rows");
    // With 512-byte key rows the operands of a whole phase would not fit the vector registers next to
    // Q, so that shape fetches and multiplies them in two halves (HV = 2); the others in one go.
    constexpr int HV = (D == 256) ? 2 : 1;
    constexpr int KSH = KS / HV;        // Q K^T MFMAs per half
    constexpr int DBH = DB / HV;        // O^T row blocks per half
    constexpr int NPVH = DBH * 2;       // P V MFMAs per half
    static_assert(KS % HV == 0 && DB % HV == 0, "halves are equal");
    constexpr int TILE_BYTES = KT * D * 2;      // bytes of a K tile and of a V^T tile in global memory
    constexpr int KROW = TileGeom<D>::KROW, VROW = TileGeom<D>::VROW;
    constexpr int K_LDS = TileGeom<D>::K_LDS, V_LDS = TileGeom<D>::V_LDS;
    constexpr int NKB = K_LDS / 1024, NVB = V_LDS / 1024;             // 1-KB wave loads per stage
    constexpr int NKI = (NKB + MFMA_WAVES - 1) / MFMA_WAVES;          // ... per wavefront (the last may be missing)
    constexpr int NVI = (NVB + MFMA_WAVES - 1) / MFMA_WAVES;
    constexpr int ATHR = 64 * MFMA_WAVES;                // threads of the work-group

    static_assert(!(SOFT && NOREF), "the soft gate keeps the running reference");
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n32 = lane & 31, hh = lane >> 5;
    int* nrflag = (int*)(ws_rw + L.off_nrflag) + blockIdx.x;
    if constexpr (NOREF) {
        if (tid == 0) *nrflag = 1;                 // unless the bound check below says otherwise
    } else if constexpr (!SOFT) {
        if (*(volatile int*)nrflag != 0) return;   // the no-reference launch before this one did the tile
    }

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

    const int rloc = wave * 32 + n32;
    const bool rvalid = rloc < S.plan.nvalid;
    const int* qperm = (const int*)(ws + L.off_qperm) + (size_t)bhq * L.NQP;
    const int qpos = rvalid ? qperm[S.plan.row0 + rloc] : -1;
    const int i_lo = S.plan.i_lo;
    const int total = S.plan.total;
    const int w = L.window;
    const int d = L.d;                  // row length of q and out
    // The allowed test of a key at position kp is one unsigned compare, (unsigned)(qadj - kp) < wlim:
    //   causal:      qadj = qpos;  wlim = 2^31 for a class that shares a group (0 <= qpos - kp), else w;
    //   non-causal:  shares a group: qadj = qpos + 2^30, wlim = 2^31 (any real key; pads sit at INT_MAX);
    //                otherwise |qpos - kp| < w: qadj = qpos + w - 1, wlim = 2w - 1.
    unsigned mq_row = 0u;
    if constexpr (COARSE) mq_row = rvalid ? ((const unsigned*)(ws + L.off_mq))[(size_t)bhq * L.n + qpos] : 0u;
    // pair_set 3 (causal): a key of a class that shares a group counts when it lies at or below qpos - w; rows whose
    // window reaches position 0 have no such key (and -1 keeps the pads, at INT_MAX, out without wrapping around)
    const int qadj_inter = L.pair_set == 3 ? max(qpos - w, -1) : L.causal ? qpos : qpos + (1 << 30);
    const int qadj_local = L.causal ? qpos : qpos + w - 1;
    const unsigned wlim_local = L.causal ? (unsigned)w : (unsigned)(2 * w - 1);
    if (total == 0) {
        // Only a launch restricted to a part of the mask can leave a tile without keys
        // (the whole mask always holds the diagonal): its rows are empty, out = 0 and lse = -inf --
        // or, in the second pass of a two-pass launch, they keep what the first pass left.
        if (rvalid && !L.merge_prev) {
            uint16_t* orow = out + (size_t)b * L.os[0] + (size_t)h * L.os[1] + (size_t)qpos * L.os[2] + hh * (d / 2);
            for (int e = 0; e < d / 2; e += 4) *(uint2*)(orow + e) = make_uint2(0u, 0u);
            if (hh == 0) {
                if (lse) lse[(size_t)bhq * L.n + qpos] = -INFINITY;
                if constexpr (PAIRS) row_pairs[(size_t)bhq * L.n + qpos] = 0;
            }
        }
        return;
    }

    V8 qreg[KS];
    {
        const V8* qrow = (const V8*)(q + (size_t)b * L.qs[0] + (size_t)h * L.qs[1] + (size_t)(rvalid ? qpos : 0) * L.qs[2]);
        V8 zero;
#pragma unroll
        for (int e = 0; e < 8; ++e) zero[e] = (elem_t)0.f;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) qreg[ks] = rvalid ? qrow[2 * ks + hh] : zero;
    }

    // Softmax without a reference (see the head of this file): every logit of row i is bounded by
    // b_i = scale*log2(e) * |q_i| * max|k| (by the cap too, with a softcap); the whole work-group needs b_i <= NOREF_BOUND.
    if constexpr (NOREF) {
        float qn2 = 0.f;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
#pragma unroll
            for (int e = 0; e < 8; ++e) qn2 = fmaf((float)qreg[ks][e], (float)qreg[ks][e], qn2);
        qn2 += __shfl_xor(qn2, 32, 64);                              // the other half of the row's components
        unsigned kn2b = ((const unsigned*)(ws + L.off_kn2))[(size_t)bhk * KN2_SLOTS + lane];
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) {
            const unsigned o = (unsigned)__shfl_xor((int)kn2b, off, 64);
            kn2b = o > kn2b ? o : kn2b;
        }
        const float kn2 = __uint_as_float(kn2b);
        float bnd = L.scale * LOG2E * NOREF_SLACK * sqrtf(qn2 * kn2);
        if constexpr (SOFTCAP) bnd = fminf(bnd, L.softcap * LOG2E);  // capped logits never leave [-cap, cap]
        if (__syncthreads_and((bnd <= NOREF_BOUND) ? 1 : 0) == 0) {  // a NaN bound compares false
            if (tid == 0) *nrflag = 0;
            return;
        }
        if constexpr (!SOFTCAP) {    // logits come off the matrix cores in log2 units
            const float sl2q = L.scale * LOG2E;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
#pragma unroll
                for (int e = 0; e < 8; ++e) qreg[ks][e] = (elem_t)((float)qreg[ks][e] * sl2q);
        }
    }

    // soft gate: this row's assignment times -lambda*log2(e), as bf16 high and low parts in B-operand order
    bf16x8 gqh[2], gql[2];
    const bool kg2 = L.K > 16;          // a second k-step of 16 groups
    if constexpr (SOFT) {
        const float* grow = g + ((size_t)b * L.n + (rvalid ? qpos : 0)) * L.K;
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int c = ks * 16 + hh * 8 + e;
                const float x = (rvalid && c < L.K) ? grow[c] * L.gate_slope : 0.f;
                const __bf16 hi = (__bf16)x;
                gqh[ks][e] = hi;
                gql[ks][e] = (__bf16)(x - (float)hi);
            }
    }

    f32x16 o[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[db][r] = 0.f;
    float m_ref = NOREF ? 0.f : -INFINITY, l_run = 0.f;
    int npairs = 0;

    const float sl2 = L.scale * LOG2E;
    const float cap_l2 = L.softcap * LOG2E;
    const float two_over_cap_l2 = (L.softcap > 0.f) ? 2.f * L.scale * LOG2E / L.softcap : 0.f;
    // cap*log2(e)*tanh(s*a), a = scale/cap, as s*(c1 + c3 s^2 + c5 s^4) while |s*a| <= CAP_POLY_Z
    const float cap_a = (L.softcap > 0.f) ? L.scale / L.softcap : 0.f;
    const float cap_c1 = L.scale * LOG2E;
    const float cap_c3 = -cap_c1 * cap_a * cap_a * (1.f / 3.f);
    const float cap_c5 = cap_c1 * cap_a * cap_a * cap_a * cap_a * (2.f / 15.f);
    const float cap_poly_lim = (L.softcap > 0.f) ? CAP_POLY_Z / cap_a : 0.f;
    const float cap_cubic_lim = (L.softcap > 0.f) ? CAP_CUBIC_Z / cap_a : 0.f;

    const char* kc_base = ws + L.off_kc + (size_t)bhk * L.NKP * (D * 2);
    const char* vt_base = ws + L.off_vt + (size_t)bhk * L.NKP * (D * 2);
    const char* kpos_base = ws + L.off_kpos + (size_t)bhk * L.NKP * 4;
    const char* kmsk_base = ws + L.off_kmsk + (size_t)bhk * L.NKP * 4;
    const char* gk_base = ws + L.off_gk + (size_t)b * L.NKP * GROW;

    // per-lane source offsets of the DMA: wave `wave` fills the 1-KB LDS blocks wave + MFMA_WAVES * i of a
    // stage; LDS byte o of a stage belongs to row o / pitch; its bytes past the row's data are padding and
    // fetch the row's last chunk again
    unsigned voff_k[NKI], voff_v[NVI];
#pragma unroll
    for (int i = 0; i < NKI; ++i) {
        const int o = (wave + MFMA_WAVES * i) * 1024 + lane * 16;
        voff_k[i] = (unsigned)((o / KROW) * (D * 2) + min(o % KROW, D * 2 - 16));
    }
#pragma unroll
    for (int i = 0; i < NVI; ++i) {
        const int o = (wave + MFMA_WAVES * i) * 1024 + lane * 16;
        voff_v[i] = (unsigned)((o / VROW) * (KT * 2) + min(o % VROW, KT * 2 - 16));
    }
    const unsigned lds_k0 = lds_addr_of(&S.k[0][0]), lds_v0 = lds_addr_of(&S.vt[0][0]);
    const unsigned lds_kp0 = lds_addr_of(&S.kpos[0][0]);
    // one address register per operand kind: this lane's row of a unit / of a 32-row block, its half-wave's chunk
    const unsigned ka_lane = lds_k0 + n32 * KROW + hh * 16;
    const unsigned va_lane = lds_v0 + n32 * VROW + hh * 16;
    const unsigned lds_km0 = lds_addr_of(&S.kmsk[0]);
    const unsigned lds_g0 = lds_addr_of(&S.gk[0]);

#define F4_DMA_K(TILE, STAGE)                                                                        \
    do {                                                                                             \
        const char* src_ = kc_base + (size_t)(TILE) * TILE_BYTES;                                    \
        _Pragma("unroll") for (int i = 0; i < NKI; ++i)                                              \
            if ((i + 1) * MFMA_WAVES <= NKB || wave + MFMA_WAVES * i < NKB)                          \
                lds_dma16(src_, voff_k[i], lds_k0 + (STAGE) * K_LDS + (wave + MFMA_WAVES * i) * 1024);   \
        if constexpr (SOFT) {            /* the keys' soft assignments travel with the key tile */          \
            const char* gsrc_ = gk_base + (size_t)(TILE) * (KT * GROW);                              \
            _Pragma("unroll") for (int i = 0; i < KT * GROW / 1024 / MFMA_WAVES; ++i)                 \
                lds_dma16(gsrc_ + (wave + MFMA_WAVES * i) * 1024, (unsigned)lane * 16, lds_g0 + (STAGE) * (KT * GROW) + (wave + MFMA_WAVES * i) * 1024); \
        }                                                                                            \
    } while (0)
#define F4_DMA_V(TILE, STAGE)                                                                        \
    do {                                                                                             \
        const char* src_ = vt_base + (size_t)(TILE) * TILE_BYTES;                                    \
        _Pragma("unroll") for (int i = 0; i < NVI; ++i)                                              \
            if ((i + 1) * MFMA_WAVES <= NVB || wave + MFMA_WAVES * i < NVB)                          \
                lds_dma16(src_, voff_v[i], lds_v0 + (STAGE) * V_LDS + (wave + MFMA_WAVES * i) * 1024);   \
    } while (0)
#define F4_DMA_KPOS(TILE, BUF)                                                                       \
    do {                                                                                             \
        if (wave == 0 && lane < KT / 4) {                                                            \
            lds_dma16(kpos_base + (size_t)(TILE) * (KT * 4), (unsigned)lane * 16, lds_kp0 + (BUF) * (KT * 4)); \
            if constexpr (COARSE)                                                                    \
                lds_dma16(kmsk_base + (size_t)(TILE) * (KT * 4), (unsigned)lane * 16, lds_km0 + (BUF) * (KT * 4)); \
        }                                                                                            \
    } while (0)
#define F4_WAIT_DMA() asm volatile("s_waitcnt vmcnt(0)" ::: "memory")

    // LDS operand reads of one unit, issued as inline asm so that they stay where they are written
    // and are NOT waited for at once: the vector work that follows runs while they are in flight,
    // and F4_WAIT_OPERANDS() (s_waitcnt lgkmcnt(0), tied to every operand register) precedes the MFMAs.
#define F4_READ_K(DST, KST, U, HALF)                                                                 \
    {                                                                                                \
        const unsigned a_ = ka_lane + (KST) * K_LDS;                                                 \
        static_for<0, KSH>([&](auto ks) {                                                            \
            DST[ks] = lds_read16_async_at<V8, (U) * 32 * KROW + ((HALF) * KSH + ks) * 32>(a_);       \
        });                                                                                          \
    }
#define F4_READ_V(DST, VST, U, HALF)                                                                 \
    {                                                                                                \
        const unsigned a_ = va_lane + (VST) * V_LDS;                                                 \
        static_for<0, NPVH>([&](auto i2) {                                                           \
            DST[i2] = lds_read16_async_at<V8, ((HALF) * DBH + i2 / 2) * 32 * VROW + (U) * 64 + (i2 % 2) * 32>(a_); \
        });                                                                                          \
    }
    // soft gate: high parts of the two k-steps, then the low parts, of the 32 keys of unit U
#define F4_READ_G(KST, U)                                                                            \
    if constexpr (SOFT) {                                                                            \
        _Pragma("unroll") for (int c = 0; c < 4; ++c) {                                              \
            const int row_ = (U) * 32 + n32;                                                         \
            ag[c] = lds_read16_async<bf16x8>(lds_g0 + (KST) * (KT * GROW) + row_ * GROW + ((((c >> 1) * 4 + (c & 1) * 2 + hh) ^ (row_ & 7)) * 16)); \
        }                                                                                            \
    }
#define F4_WAIT_OPERANDS()                                                                           \
    wait_lds_operands(ak);                                                                           \
    pin_operands(av);                                                                                \
    if constexpr (SOFT) pin_operands(ag);
    // G^T of one unit: (high x high) + (high x low) + (low x high) per k-step of 16 groups
#define F4_GATE_MFMAS(GOUT)                                                                          \
    if constexpr (SOFT) {                                                                            \
        _Pragma("unroll") for (int r = 0; r < 16; ++r) GOUT[r] = 0.f;                                \
        GOUT = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ag[0], gqh[0], GOUT, 0, 0, 0);                \
        GOUT = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ag[0], gql[0], GOUT, 0, 0, 0);                \
        GOUT = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ag[2], gqh[0], GOUT, 0, 0, 0);                \
        if (kg2) {                                                                                   \
            GOUT = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ag[1], gqh[1], GOUT, 0, 0, 0);            \
            GOUT = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ag[1], gql[1], GOUT, 0, 0, 0);            \
            GOUT = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ag[3], gqh[1], GOUT, 0, 0, 0);            \
        }                                                                                            \
    }

    // Scalar walk over the tile sequence (class by class).  A tile travels as one packed word:
    // bits 0..29 tile index, bit 30 "class shares a group" flag, bit 31 "no mask needed" flag.
    // LDS is touched only when the walk enters a new class; past the end the last tile repeats.
    int w_c = -1, w_t = 0, w_end = 0, w_int_beg = 0, w_int_end = 0, w_flag = 0, w_last = 0;
    auto next_tile = [&]() -> unsigned {
        if (w_t >= w_end) {
            int c = w_c + 1;
            while (c < L.NC && S.plan.cum[c + 1] == S.plan.cum[c]) ++c;
            if (c < L.NC) {
                w_c = __builtin_amdgcn_readfirstlane(c);
                w_t = __builtin_amdgcn_readfirstlane(S.plan.t0[c]);
                w_end = w_t + __builtin_amdgcn_readfirstlane(S.plan.cum[c + 1] - S.plan.cum[c]);
                w_int_beg = __builtin_amdgcn_readfirstlane(S.plan.ibeg[c]);
                w_int_end = __builtin_amdgcn_readfirstlane(S.plan.iend[c]);
                w_flag = __builtin_amdgcn_readfirstlane((int)S.plan.inter[c]) << 30;
            } else {
                return (unsigned)w_last;                      // sequence exhausted
            }
        }
        w_last = w_t | w_flag | ((w_t >= w_int_beg && w_t < w_int_end) ? (int)0x80000000u : 0);
        ++w_t;
        return (unsigned)w_last;
    };
    constexpr unsigned TILE_MASK = 0x3fffffffu;

    // ---- prologue: K(0), V(0) -> stage 0; K(1) -> stage 1; kpos(0), kpos(1); zero V stage 1
    unsigned pk0, pk1, pk2;                                  // packed tiles t, t+1, t+2
    {
        pk0 = next_tile();
        pk1 = next_tile();
        pk2 = next_tile();
        const int t0 = (int)(pk0 & TILE_MASK), t1 = (int)(pk1 & TILE_MASK);
        F4_DMA_K(t0, 0);
        F4_DMA_V(t0, 0);
        F4_DMA_K(t1, 1);
        F4_DMA_KPOS(t0, 0);
        F4_DMA_KPOS(t1, 1);
        const u32x4 z4 = {0u, 0u, 0u, 0u};
        for (int i = tid; i < V_LDS / 16; i += ATHR) *(u32x4*)(S.vt[1] + i * 16) = z4;
        F4_WAIT_DMA();
    }
    __syncthreads();
    f32x16 s0, s1;
    V8 p0[2], p1[2];
    V2 ones2;
    ones2[0] = (elem_t)1.0f;
    ones2[1] = (elem_t)1.0f;
    V8 ak[KSH], av[NPVH];
    bf16x8 ag[4];
    f32x16 g0acc, g1acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) { s0[r] = 0.f; s1[r] = 0.f; g0acc[r] = 0.f; g1acc[r] = 0.f; }
#pragma unroll
    for (int e = 0; e < 8; ++e) { p1[0][e] = (elem_t)0.f; p1[1][e] = (elem_t)0.f; p0[0][e] = (elem_t)0.f; p0[1][e] = (elem_t)0.f; }
    {
        F4_READ_K(ak, 0, 0, 0)
        F4_READ_G(0, 0)
        wait_lds_operands(ak);
        if constexpr (SOFT) pin_operands(ag);
#pragma unroll
        for (int ks = 0; ks < KSH; ++ks) s0 = HT::mfma(ak[ks], qreg[ks], s0);
        F4_GATE_MFMAS(g0acc)
    }
    if constexpr (HV == 2) {
        F4_READ_K(ak, 0, 0, 1)
        wait_lds_operands(ak);
#pragma unroll
        for (int ks = 0; ks < KSH; ++ks) s0 = HT::mfma(ak[ks], qreg[KSH + ks], s0);
    }

    // softmax step on one unit's scores: SIN (f32x16, consumed) -> POUT (2 x bf16x8), split in two parts.
    // PPEND: probabilities of the previous unit whose PV product has not been issued yet.
    // NOREF: no row max, no rescaling, exp2 of the logit itself.
#define F4_SOFTMAX_PRE(SIN, U, KPB, PPEND, GIN)                                                          \
    if constexpr (SOFT) {                                                                                \
        /* Eq. 2: score * (local ? 1 : sigmoid(lambda g_i.g_j)), then the causal mask (pads sit at INT_MAX) */ \
        if (far_) {                      /* the whole tile lies before every row's window: gate only */  \
            _Pragma("unroll") for (int r = 0; r < 16; ++r)                                               \
                SIN[r] *= __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(GIN[r]));                   \
        } else                                                                                           \
        _Pragma("unroll") for (int r4 = 0; r4 < 4; ++r4) {                                               \
            const int4 kp4_ = *(const int4*)(&S.kpos[KPB][(U) * 32 + 8 * r4 + 4 * hh]);                  \
            const int kp_[4] = {kp4_.x, kp4_.y, kp4_.z, kp4_.w};                                         \
            _Pragma("unroll") for (int e = 0; e < 4; ++e) {                                              \
                const unsigned dlt_ = (unsigned)(qpos - kp_[e]);                                         \
                const float gate_ = __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(GIN[r4 * 4 + e])); \
                const float sg_ = SIN[r4 * 4 + e] * ((dlt_ < (unsigned)w) ? 1.f : gate_);                \
                SIN[r4 * 4 + e] = (dlt_ < 0x80000000u) ? sg_ : -INFINITY;                                \
            }                                                                                            \
        }                                                                                                \
    } else                                                                                               \
    if constexpr (SOFTCAP) {                                                                             \
        /* cap*tanh(z), z = s*scale/cap.  While every |z| of the unit is below CAP_POLY_Z the odd Taylor */ \
        /* polynomial to z^5 stands in for tanh (error below 17 z^7 / 315: 6e-4 in the logit at cap 50, */ \
        /* under the rounding of the 16-bit probabilities): four plain instructions per score instead   */ \
        /* of an exp2 and a reciprocal.  Otherwise the exact form 1 - 2 / (1 + e^(2z)).  The 8-wavefront */ \
        /* instantiations that do not count pairs (long sequences; the others have no register to spare) */ \
        /* also drop the z^5 term while every |z| of the unit is below CAP_CUBIC_Z: three instructions.  */ \
        float am_ = fabsf(SIN[0]);                                                                       \
        _Pragma("unroll") for (int r = 1; r < 16; ++r) am_ = fmaxf(am_, fabsf(SIN[r]));                  \
        if (__any(!(am_ <= cap_poly_lim))) {                                                             \
            _Pragma("unroll") for (int r = 0; r < 16; ++r) {                                             \
                const float e2_ = __builtin_amdgcn_exp2f(SIN[r] * two_over_cap_l2);                      \
                SIN[r] = cap_l2 - 2.f * cap_l2 * __builtin_amdgcn_rcpf(1.f + e2_);                       \
            }                                                                                            \
        } else if (PAIRS || COARSE || MFMA_WAVES != 8 || __any(!(am_ <= cap_cubic_lim))) {               \
            _Pragma("unroll") for (int r = 0; r < 16; ++r) {                                             \
                const float u_ = SIN[r] * SIN[r];                                                        \
                SIN[r] *= fmaf(fmaf(u_, cap_c5, cap_c3), u_, cap_c1);                                    \
            }                                                                                            \
        } else {                                                                                         \
            _Pragma("unroll") for (int r = 0; r < 16; ++r)                                               \
                SIN[r] *= fmaf(SIN[r] * SIN[r], cap_c3, cap_c1);                                         \
        }                                                                                                \
    }                                                                                                    \
    if (SOFT) {                          /* masked above */                                              \
    } else if (!interior) {                                                                              \
        _Pragma("unroll") for (int r4 = 0; r4 < 4; ++r4) {                                               \
            const int4 kp4_ = *(const int4*)(&S.kpos[KPB][(U) * 32 + 8 * r4 + 4 * hh]);                  \
            const int kp_[4] = {kp4_.x, kp4_.y, kp4_.z, kp4_.w};                                         \
            unsigned km_[4] = {0u, 0u, 0u, 0u};                                                          \
            if constexpr (COARSE) {                                                                      \
                const uint4 km4_ = *(const uint4*)(&S.kmsk[(KPB) * KT + (U) * 32 + 8 * r4 + 4 * hh]);    \
                km_[0] = km4_.x; km_[1] = km4_.y; km_[2] = km4_.z; km_[3] = km4_.w;                      \
            }                                                                                            \
            _Pragma("unroll") for (int e = 0; e < 4; ++e) {                                              \
                bool ok_ = (unsigned)(qadj - kp_[e]) < wlim;                                             \
                if constexpr (COARSE) {                                                                  \
                    /* a common super-group only: the pair needs a common group or the window; a launch */ \
                    /* restricted to one pair set keeps the pairs with a common group, or the local rest */ \
                    if (shares_) {                                                                       \
                        const bool sh_ = (mq_row & km_[e]) != 0u;                                        \
                        const bool loc_ = (unsigned)(qadj_local - kp_[e]) < wlim_local;                  \
                        ok_ = ok_ && (L.pair_set == 1 ? sh_ : L.pair_set == 2 ? (loc_ && !sh_) : (sh_ || loc_)); \
                    }                                                                                    \
                }                                                                                        \
                SIN[r4 * 4 + e] = ok_ ? SIN[r4 * 4 + e] : -INFINITY;                                     \
                if constexpr (PAIRS) npairs += ok_ ? 1 : 0;                                              \
            }                                                                                            \
        }                                                                                                \
    } else {                                                                                             \
        if constexpr (PAIRS) npairs += 16;                                                               \
    }                                                                                                    \
    if (!NOREF) {                                                                                        \
        float mx_ = SIN[0];                                                                              \
        _Pragma("unroll") for (int r = 1; r < 16; ++r) mx_ = fmaxf(mx_, SIN[r]);                         \
        mx_ = halfwave_max(mx_);                                                                         \
        const float m2_ = SOFTCAP ? mx_ : mx_ * sl2;                                                     \
        const bool upd_ = m2_ > m_ref + RESCALE_THRESHOLD;                                               \
        if (__any(upd_)) {                                                                               \
            const float alpha_ = upd_ ? __builtin_amdgcn_exp2f(m_ref - m2_) : 1.f;                       \
            m_ref = upd_ ? m2_ : m_ref;                                                                  \
            l_run *= alpha_;                                                                             \
            _Pragma("unroll") for (int db = 0; db < DB; ++db)                                            \
                _Pragma("unroll") for (int r = 0; r < 16; ++r) o[db][r] *= alpha_;                       \
            /* probabilities still waiting for their PV product were taken against the old reference */ \
            _Pragma("unroll") for (int e = 0; e < 8; ++e) {                                              \
                PPEND[0][e] = (elem_t)((float)PPEND[0][e] * alpha_);                                     \
                PPEND[1][e] = (elem_t)((float)PPEND[1][e] * alpha_);                                     \
            }                                                                                            \
        }                                                                                                \
    }
#define F4_SOFTMAX_EXP(SIN, POUT)                                                                        \
    {                                                                                                    \
        const float m_use_ = NOREF ? 0.f : (m_ref == -INFINITY) ? 0.f : m_ref;                           \
        float psum_ = 0.f;                                                                               \
        _Pragma("unroll") for (int r = 0; r < 16; r += 2) {                                              \
            const float a0_ = NOREF ? SIN[r] : SOFTCAP ? (SIN[r] - m_use_) : fmaf(SIN[r], sl2, -m_use_); \
            const float a1_ = NOREF ? SIN[r + 1] : SOFTCAP ? (SIN[r + 1] - m_use_) : fmaf(SIN[r + 1], sl2, -m_use_); \
            V2 pr_;                                                                                      \
            pr_[0] = (elem_t)((FOCUS_ABLATE & 2) ? a0_ : __builtin_amdgcn_exp2f(a0_));                   \
            pr_[1] = (elem_t)((FOCUS_ABLATE & 2) ? a1_ : __builtin_amdgcn_exp2f(a1_));                   \
            /* the row sum adds the ROUNDED probabilities, the same numbers the PV product uses */      \
            psum_ = HT::dot2(pr_, ones2, psum_);                                                         \
            POUT[r / 8][r % 8] = pr_[0];                                                                 \
            POUT[r / 8][r % 8 + 1] = pr_[1];                                                             \
        }                                                                                                \
        l_run += psum_;                                                                                  \
    }
    // the MFMAs of (one half of) a phase: PV with pending probabilities PP, then the QK^T unit into SOUT
#define F4_MFMAS(PP, SOUT, HALF, GOUT)                                                                   \
    if ((HALF) == 0) { F4_GATE_MFMAS(GOUT) }                                                             \
    _Pragma("unroll") for (int i = 0; i < NPVH; ++i)                                                     \
        o[(HALF) * DBH + i / 2] = HT::mfma(av[i], PP[i % 2], o[(HALF) * DBH + i / 2]);                   \
    if ((HALF) == 0) { _Pragma("unroll") for (int r = 0; r < 16; ++r) SOUT[r] = 0.f; }                   \
    _Pragma("unroll") for (int ks = 0; ks < KSH; ++ks)                                                   \
        SOUT = HT::mfma(ak[ks], qreg[(HALF) * KSH + ks], SOUT);
    // keeps values computed / loaded where they are written in the source (no sinking past a branch)
#define F4_PIN2(P_) asm volatile("" : "+v"(P_[0]), "+v"(P_[1]))
    int kb_cur = 0;                                          // kpos buffer of tile t (t mod 3)
    // One key tile.  SC is the LDS stage of K(t), V(t); K(t+1), V(t-1) sit in the other.
#if (FOCUS_ABLATE & 8)
#undef F4_READ_K
#undef F4_READ_V
#define F4_READ_K(DST, KST, U, HALF) { asm volatile("" : "+v"(DST[0])); }
#define F4_READ_V(DST, VST, U, HALF) { asm volatile("" : "+v"(DST[0])); }
#endif
#define F4_TILE(SC)                                                                                      \
    {                                                                                                    \
        const int sc = (SC), sn = (SC) ^ 1;                                                              \
        const bool shares_ = ((pk0 >> 30) & 1u) != 0;        /* the key class shares a group with the rows */ \
        const unsigned wlim = shares_ ? 0x80000000u : wlim_local;                                        \
        const int qadj = shares_ ? qadj_inter : qadj_local;                                              \
        const bool interior = (pk0 >> 31) != 0;                                                          \
        /* soft gate, position order: keys of this tile all at or below i_lo - w (and real, and causal) */ \
        const bool far_ = SOFT && interior && ((int)(pk0 & TILE_MASK) * KT + KT - 1 + w <= i_lo);        \
        const int tl1 = (int)(pk1 & TILE_MASK);                                                          \
        const int tl2 = (int)(pk2 & TILE_MASK);                                                          \
        const int kb_nn = (kb_cur >= 1) ? kb_cur - 1 : 2;    /* (t+2) mod 3 */                           \
        /* phase A: VALU softmax(S0) -> P0 ; MFMA O += V(t-1,u1) P1 and S1 = K(t,u1) Q^T */              \
        F4_READ_V(av, sn, 1, 0)                                                                          \
        F4_READ_K(ak, sc, 1, 0)                                                                          \
        F4_READ_G(sc, 1)                                                                                 \
        F4_SOFTMAX_PRE(s0, 0, kb_cur, p1, g0acc)                                                         \
        F4_WAIT_OPERANDS()                                                                               \
        F4_MFMAS(p1, s1, 0, g1acc)                                                                       \
        if constexpr (HV == 2) {                                                                         \
            F4_READ_V(av, sn, 1, 1)                                                                      \
            F4_READ_K(ak, sc, 1, 1)                                                                      \
        }                                                                                                \
        F4_SOFTMAX_EXP(s0, p0)                                                                           \
        if constexpr (HV == 2) {                                                                         \
            F4_WAIT_OPERANDS()                                                                           \
            F4_MFMAS(p1, s1, 1, g1acc)                                                                   \
        }                                                                                                \
        __builtin_amdgcn_iglp_opt(3);                                                                    \
        F4_PIN2(p0);                                                                                     \
        /* one barrier per tile: all are done with K(t), V(t-1); K(t+1), V(t) have landed */             \
        if (!(FOCUS_ABLATE & 16)) F4_WAIT_DMA();                                                         \
        if (!(FOCUS_ABLATE & 1)) __syncthreads();                                                        \
        if (!(FOCUS_ABLATE & 4)) {                                                                       \
            F4_DMA_K(tl2, sc);                                                                           \
            F4_DMA_V(tl1, sn);                                                                           \
            F4_DMA_KPOS(tl2, kb_nn);                                                                     \
        }                                                                                                \
        /* phase B: VALU softmax(S1) -> P1 ; MFMA O += V(t,u0) P0 and S0 = K(t+1,u0) Q^T */              \
        F4_READ_V(av, sc, 0, 0)                                                                          \
        F4_READ_K(ak, sn, 0, 0)                                                                          \
        F4_READ_G(sn, 0)                                                                                 \
        F4_SOFTMAX_PRE(s1, 1, kb_cur, p0, g1acc)                                                         \
        F4_WAIT_OPERANDS()                                                                               \
        F4_MFMAS(p0, s0, 0, g0acc)                                                                       \
        if constexpr (HV == 2) {                                                                         \
            F4_READ_V(av, sc, 0, 1)                                                                      \
            F4_READ_K(ak, sn, 0, 1)                                                                      \
        }                                                                                                \
        F4_SOFTMAX_EXP(s1, p1)                                                                           \
        if constexpr (HV == 2) {                                                                         \
            F4_WAIT_OPERANDS()                                                                           \
            F4_MFMAS(p0, s0, 1, g0acc)                                                                   \
        }                                                                                                \
        __builtin_amdgcn_iglp_opt(3);                                                                    \
        F4_PIN2(p1);                                                                                     \
        kb_cur = (kb_cur == 2) ? 0 : kb_cur + 1;                                                         \
        pk0 = pk1;                                                                                       \
        pk1 = pk2;                                                                                       \
        pk2 = next_tile();                                                                               \
    }
    for (int it = 0; it < total; ++it) {
        F4_TILE(it & 1)
    }
#undef F4_TILE
    // ---- drain: O += V(T-1,u1) P1 (V(T-1) was complete before the last barrier)
    {
        const int sl = (total - 1) & 1;
        {
            F4_READ_V(av, sl, 1, 0)
            wait_lds_operands(av);
#pragma unroll
            for (int i = 0; i < NPVH; ++i) o[i / 2] = HT::mfma(av[i], p1[i % 2], o[i / 2]);
        }
        if constexpr (HV == 2) {
            F4_READ_V(av, sl, 1, 1)
            wait_lds_operands(av);
#pragma unroll
            for (int i = 0; i < NPVH; ++i) o[DBH + i / 2] = HT::mfma(av[i], p1[i % 2], o[DBH + i / 2]);
        }
    }
    F4_WAIT_DMA();                                           // nothing may still be writing LDS when the block ends
#undef F4_DMA_K
#undef F4_DMA_V
#undef F4_DMA_KPOS
#undef F4_WAIT_DMA
#undef F4_READ_K
#undef F4_READ_V
#undef F4_SOFTMAX_PRE
#undef F4_SOFTMAX_EXP
#undef F4_MFMAS
#undef F4_PIN2
#undef F4_WAIT_OPERANDS
#undef F4_READ_G
#undef F4_GATE_MFMAS

    // ---- epilogue
    const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
    if constexpr (PAIRS) npairs += __shfl_xor(npairs, 32, 64);
    if (!rvalid) return;
    float inv = (l_tot > 0.f) ? 1.f / l_tot : 0.f;            // an empty row (restricted pair set): out = 0, lse = -inf
    uint16_t* orow = out + (size_t)b * L.os[0] + (size_t)h * L.os[1] + (size_t)qpos * L.os[2];
    // Second pass of a two-pass launch: this row's result over the pairs inside the window is in out / lse
    // (16-bit, natural log).  out = (e^{l1} o1 + e^{l2} o2) / (e^{l1} + e^{l2}), App. D's merge, in log2 units.
    float w1 = 0.f, lse2_l2 = m_ref + __builtin_amdgcn_logf(l_tot);      // -inf for an empty row
    if (L.merge_prev) {
        if (!(l_tot > 0.f)) return;                           // nothing outside the window: the first pass stands
        const float lse1_l2 = lse[(size_t)bhq * L.n + qpos] * LOG2E;
        const float top = fmaxf(lse1_l2, lse2_l2);
        w1 = __builtin_amdgcn_exp2f(lse1_l2 - top);
        const float w2 = __builtin_amdgcn_exp2f(lse2_l2 - top);
        const float den = 1.f / (w1 + w2);
        inv *= w2 * den;
        w1 *= den;
        lse2_l2 = top + __builtin_amdgcn_logf(w1 / den + w2);
    }
#pragma unroll
    for (int db = 0; db < DB; ++db) {
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
            const int dcol = db * 32 + 8 * r4 + 4 * hh;
            if (DB * 32 > KS * 16 && dcol >= d) continue;        // rows of O^T past a head dim that is no multiple of 32
            float f0 = o[db][r4 * 4 + 0] * inv, f1 = o[db][r4 * 4 + 1] * inv;
            float f2 = o[db][r4 * 4 + 2] * inv, f3 = o[db][r4 * 4 + 3] * inv;
            if (L.merge_prev) {
                const uint2 prev = *(const uint2*)(orow + dcol);
                elem_t p0_, p1_, p2_, p3_;
                const uint16_t b0 = (uint16_t)(prev.x & 0xffffu), b1 = (uint16_t)(prev.x >> 16);
                const uint16_t b2 = (uint16_t)(prev.y & 0xffffu), b3 = (uint16_t)(prev.y >> 16);
                __builtin_memcpy(&p0_, &b0, 2); __builtin_memcpy(&p1_, &b1, 2);
                __builtin_memcpy(&p2_, &b2, 2); __builtin_memcpy(&p3_, &b3, 2);
                f0 = fmaf(w1, (float)p0_, f0); f1 = fmaf(w1, (float)p1_, f1);
                f2 = fmaf(w1, (float)p2_, f2); f3 = fmaf(w1, (float)p3_, f3);
            }
            elem_t e0 = (elem_t)f0, e1 = (elem_t)f1, e2 = (elem_t)f2, e3 = (elem_t)f3;
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
        if (lse) lse[(size_t)bhq * L.n + qpos] = lse2_l2 * (1.f / LOG2E);
        if constexpr (PAIRS) row_pairs[(size_t)bhq * L.n + qpos] = npairs + (L.merge_prev ? row_pairs[(size_t)bhq * L.n + qpos] : 0);
    }
}

template <int D, int KS, int DB, int WAVES, bool SOFTCAP, bool PAIRS, bool F16, bool COARSE, bool SOFT = false>
hipError_t launch_one(const Layout& L, const HeadMap& hm, int default_map, const void* q, char* ws, void* out,
                      float* lse, int32_t* row_pairs, hipStream_t st, const float* g = nullptr)
{
    const unsigned grid = (unsigned)((size_t)L.NT * L.B * L.Hq);
    if constexpr (!SOFT)
        hipLaunchKernelGGL((attn_mfma_kernel<D, KS, DB, WAVES, SOFTCAP, PAIRS, F16, COARSE, SOFT, true>), dim3(grid),
                           dim3(64 * WAVES), 0, st, L, hm, default_map, (const uint16_t*)q, g, ws, (uint16_t*)out, lse,
                           row_pairs);
    hipLaunchKernelGGL((attn_mfma_kernel<D, KS, DB, WAVES, SOFTCAP, PAIRS, F16, COARSE, SOFT, false>), dim3(grid),
                       dim3(64 * WAVES), 0, st, L, hm, default_map, (const uint16_t*)q, g, ws, (uint16_t*)out, lse,
                       row_pairs);
    return hipGetLastError();
}

template <int D, int KS, int DB, int WAVES, bool F16, bool COARSE>
hipError_t launch_w(const Layout& L, const HeadMap& hm, int default_map, const void* q, char* ws, void* out,
                    float* lse, int32_t* row_pairs, hipStream_t st)
{
    const bool sc = L.softcap > 0.f, pairs = row_pairs != nullptr;
    if (sc) {
        return pairs ? launch_one<D, KS, DB, WAVES, true, true, F16, COARSE>(L, hm, default_map, q, ws, out, lse, row_pairs, st)
                     : launch_one<D, KS, DB, WAVES, true, false, F16, COARSE>(L, hm, default_map, q, ws, out, lse, row_pairs, st);
    }
    return pairs ? launch_one<D, KS, DB, WAVES, false, true, F16, COARSE>(L, hm, default_map, q, ws, out, lse, row_pairs, st)
                 : launch_one<D, KS, DB, WAVES, false, false, F16, COARSE>(L, hm, default_map, q, ws, out, lse, row_pairs, st);
}

template <int D, int KS, int DB>
hipError_t launch_d(const Layout& L, const HeadMap& hm, int default_map, const void* q, const void* v, const float* g,
                    char* ws, void* out, float* lse, int32_t* row_pairs, hipStream_t st)
{
    dim3 ggrid(L.NKP / KT, L.B * L.Hkv);
    hipLaunchKernelGGL(gather_vt_kernel<D>, ggrid, dim3(NTHR), 0, st, L, (const uint16_t*)v, ws);
    const bool f16 = L.dtype == 2;
    if (L.soft) {                        // 128-row tiles, no softcap, no pair counts (a row i attends i + 1 keys)
        if (L.BQ != 128 || !g || row_pairs || L.softcap > 0.f) return hipErrorInvalidValue;
        // 512-byte key rows plus the gate's accumulators and operands do not fit the register file
        if constexpr (D == 256) return hipErrorInvalidValue;
        else
        return f16 ? launch_one<D, KS, DB, 4, false, false, true, false, true>(L, hm, default_map, q, ws, out, lse, nullptr, st, g)
                   : launch_one<D, KS, DB, 4, false, false, false, false, true>(L, hm, default_map, q, ws, out, lse, nullptr, st, g);
    }
    // the query tile size fixed by focus_assign selects the work-group shape: 4 or 8 wavefronts
    if constexpr (D != 256) {
        if (L.BQ == 256)
            return f16 ? launch_w<D, KS, DB, 8, true, false>(L, hm, default_map, q, ws, out, lse, row_pairs, st)
                       : launch_w<D, KS, DB, 8, false, false>(L, hm, default_map, q, ws, out, lse, row_pairs, st);
    }
    if (L.BQ != 128) return hipErrorInvalidValue;
    if (L.coarse)                        // coarse classes always use 128-row tiles
        return f16 ? launch_w<D, KS, DB, 4, true, true>(L, hm, default_map, q, ws, out, lse, row_pairs, st)
                   : launch_w<D, KS, DB, 4, false, true>(L, hm, default_map, q, ws, out, lse, row_pairs, st);
    return f16 ? launch_w<D, KS, DB, 4, true, false>(L, hm, default_map, q, ws, out, lse, row_pairs, st)
               : launch_w<D, KS, DB, 4, false, false>(L, hm, default_map, q, ws, out, lse, row_pairs, st);
}

}  // namespace

// the soft assignments of the key positions as the matrix cores read them (see Layout::off_gk)
__global__ __launch_bounds__(256) void soft_gather_g_kernel(Layout L, const float* __restrict__ g, char* __restrict__ ws)
{
    const size_t total = (size_t)L.B * L.NKP * 8;         // 16-byte chunks: 4 of high parts, 4 of low parts per key
    for (size_t id = (size_t)blockIdx.x * blockDim.x + threadIdx.x; id < total; id += (size_t)gridDim.x * blockDim.x) {
        const int c8 = (int)(id % 8);
        const size_t slot = (id / 8) % L.NKP;             // one class in position order: slot = position, pads after n
        const size_t b = id / 8 / L.NKP;
        const int part = c8 / 4, e0 = (c8 % 4) * 8;
        uint16_t h[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int c = e0 + e;
            const float x = (slot < (size_t)L.n && c < L.K) ? g[(b * L.n + slot) * L.K + c] : 0.f;
            const __bf16 hi = (__bf16)x;
            const __bf16 val = part ? (__bf16)(x - (float)hi) : hi;
            __builtin_memcpy(&h[e], &val, 2);
        }
        uint4 u;
        u.x = h[0] | ((uint32_t)h[1] << 16); u.y = h[2] | ((uint32_t)h[3] << 16);
        u.z = h[4] | ((uint32_t)h[5] << 16); u.w = h[6] | ((uint32_t)h[7] << 16);
        // chunks swizzled inside a key's 128 bytes so that 8 consecutive keys spread over the LDS banks
        *(uint4*)(ws + L.off_gk + (b * L.NKP + slot) * GROW + (size_t)((c8 ^ (int)(slot & 7)) * 16)) = u;
    }
}

hipError_t launch_soft_gather_g(const Layout& L, const float* g, char* ws, hipStream_t st)
{
    const size_t total = (size_t)L.B * L.NKP * 8;
    const unsigned grid = (unsigned)std::min<size_t>(8192, (total + 255) / 256);
    hipLaunchKernelGGL(soft_gather_g_kernel, dim3(grid), dim3(256), 0, st, L, g, ws);
    return hipGetLastError();
}

hipError_t launch_attn_mfma(const Layout& L, const HeadMap& hm, const void* q, const void* k, const void* v,
                            const float* g, char* ws, void* out, float* lse, int32_t* row_pairs, hipStream_t st)
{
    (void)k;
    int default_map = 1;
    const int G = L.Hq / L.Hkv;
    if (L.Hq % L.Hkv != 0) default_map = 0;
    else
        for (int h = 0; h < L.Hq; ++h)
            if (hm.kv[h] != h / G) default_map = 0;
    if ((size_t)L.NT * L.B * L.Hq > 0x7fffffffull) return hipErrorInvalidValue;
    switch (L.d) {
        case 64: return launch_d<64, 4, 2>(L, hm, default_map, q, v, g, ws, out, lse, row_pairs, st);
        case 80: return launch_d<128, 5, 3>(L, hm, default_map, q, v, g, ws, out, lse, row_pairs, st);
        case 96: return launch_d<128, 6, 3>(L, hm, default_map, q, v, g, ws, out, lse, row_pairs, st);
        case 128: return launch_d<128, 8, 4>(L, hm, default_map, q, v, g, ws, out, lse, row_pairs, st);
        case 256: return launch_d<256, 16, 8>(L, hm, default_map, q, v, g, ws, out, lse, row_pairs, st);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace focus
