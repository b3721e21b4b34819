// focus_assign: centroid scoring, top-k membership, bucketing by group and by
// membership class (Sec. 2 Eq. 1 in per-head dot-product form; Sec. 2
// "Efficiency at inference"; the stable sort by group of App. D done as a
// counting sort).
//
// Four launches per focus_assign call, the work item everywhere a (sort block of
// SB positions, batch*head) pair:
//   assign_init  centroids to fp64, the key-norm slots to zero (a few us);
//   score_topk   streams q (or k) once, scores every token against the K centroids of its KV
//                head in fp64 (products are exact in fp64, added in index order,
//                so the result is reproducible bit for bit), keeps the top-k
//                groups, writes the membership mask, the class id and the
//                per-block histograms of classes and groups;
//   scan_plan    one work-group per (batch, head) row: exclusive scan of the
//                row's histograms over the sort blocks, then class offsets
//                (padded to tile multiples), group list offsets, the class ->
//                group-mask table and the job list of query tiles;
//   scatter      stable ranks inside a block by wavefront ballot + popcount,
//                coalesced 4-byte writes of the class-ordered position arrays
//                and of the per-group index lists, the pads of those arrays, and
//                (key rows, 16-bit types) the class-ordered copy of the key rows
//                with the largest squared key norm of the head.
// Memberships given per token (focus_assign_tokens) take token_classes in place
// of score_topk.
#include "focus_internal.h"
#include <hip/hip_bf16.h>
#include <algorithm>
#include <type_traits>

namespace focus {

namespace {

__device__ inline float bf16_bits_to_f32(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

// Pascal's triangle up to C(32, .), built at compile time: the class of a token is the colex rank of
// its membership set, a sum of binomials.
struct BinomTable { uint32_t v[33 * 33]; };
constexpr BinomTable make_binom_table()
{
    BinomTable t{};
    for (int a = 0; a <= 32; ++a) {
        for (int b = 0; b <= 32; ++b) {
            uint32_t x = 0;
            if (b == 0 || b == a) x = (b <= a) ? 1u : 0u;
            else if (b < a) x = t.v[(a - 1) * 33 + b - 1] + t.v[(a - 1) * 33 + b];
            t.v[a * 33 + b] = x;
        }
    }
    return t;
}
__device__ __constant__ BinomTable g_binom = make_binom_table();

// ---------------------------------------------------------------- score + top-k
constexpr int ROW_CHUNK_BYTES = 128;                 // bytes of every row staged per phase
constexpr int ROW_STRIDE = ROW_CHUNK_BYTES + 16;     // padded LDS row stride


typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// The kernels of the bucketing serve the query side, the key side, or both in one launch (which = 1, 0, -1):
// with both, the rows [0, B*Hq) of the launch are query (batch, head) pairs and the B*Hkv after them key pairs.
constexpr int MAX_GRID_ROWS = 65535;
__device__ inline int side_of_row(const Layout& L, int which, unsigned row) { return which < 0 ? (int)(row < (unsigned)(L.B * L.Hq)) : which; }
__device__ inline int row_in_side(const Layout& L, int which, unsigned row)
{
    return (which < 0 && row >= (unsigned)(L.B * L.Hq)) ? (int)row - L.B * L.Hq : (int)row;
}

// ---------------------------------------------------------------- scan over sort blocks + per-row plan
// One (batch, head) row, all NTHREADS threads of a work-group: exclusive scan of every histogram column over
// the sort blocks (in place, total in row nblk), then class offsets (padded to tile multiples), group list
// offsets, the class -> group-mask table (first query row) and the job list of the query tiles.
// The histograms pass through LDS a chunk of sort blocks at a time.  tmp: tmp_ints >= SCAN_PLAN_FIXED_INTS + NC + K ints of LDS.

constexpr int SCAN_THREADS = 1024;                                   // threads of the scan + plan work-group
constexpr int SCAN_PLAN_FIXED_INTS = SCAN_THREADS + 2 * MAX_CLASSES + 40;   // s_part, s_tot, s_nt, s_total
constexpr int SCAN_PLAN_TMP_INTS = 9216;                             // 36 KB of LDS
static_assert(SCAN_PLAN_TMP_INTS >= SCAN_PLAN_FIXED_INTS + MAX_CLASSES + 32, "room for at least one sort block");

template <int NTHREADS>
__device__ inline void scan_and_plan_row(const Layout& L, int is_query, int bh, char* __restrict__ ws, int* tmp, int tmp_ints)
{
    const int tid = threadIdx.x;
    const int NC = L.NC, K = L.K, nblk = L.nblk;
    int* s_part = tmp;                          // [NTHREADS] partial sums of the scan
    int* s_tot = tmp + NTHREADS;                // [NC + K] running column totals
    int* s_nt = s_tot + MAX_CLASSES + 32;       // [NC] query tiles per class
    int* s_total = s_nt + MAX_CLASSES;          // [1]
    int* stage = tmp + SCAN_PLAN_FIXED_INTS;    // histograms of a chunk of sort blocks, [blocks][NC + K]
    int* bc_base = (int*)(ws + (is_query ? L.off_qbc : L.off_kbc)) + (size_t)bh * (nblk + 1) * NC;
    int* bg_base = (int*)(ws + (is_query ? L.off_qbg : L.off_kbg)) + (size_t)bh * (nblk + 1) * K;
    const int ncol = NC + K;
    const int cb = max(1, min(nblk, (tmp_ints - SCAN_PLAN_FIXED_INTS) / ncol));   // sort blocks per chunk
    const int cpp = min(ncol, NTHREADS);        // columns per pass
    const int P = NTHREADS / cpp;               // threads per column: each scans a run of the chunk's blocks
    for (int c = tid; c < ncol; c += NTHREADS) s_tot[c] = 0;
    for (int b0 = 0; b0 < nblk; b0 += cb) {
        const int nb = min(cb, nblk - b0);
        const int ne = nb * ncol;
        __syncthreads();                        // the previous chunk's stage is no longer read; s_tot is set
        // the chunk into LDS, eight independent loads in flight per thread
        for (int e0 = 0; e0 < ne; e0 += 8 * NTHREADS) {
            int v[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int e = e0 + i * NTHREADS + tid;
                v[i] = 0;
                if (e < ne) {
                    const int b = b0 + e / ncol, c = e % ncol;
                    v[i] = c < NC ? bc_base[(size_t)b * NC + c] : bg_base[(size_t)b * K + (c - NC)];
                }
            }
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int e = e0 + i * NTHREADS + tid;
                if (e < ne) stage[e] = v[i];
            }
        }
        __syncthreads();
        const int run = (nb + P - 1) / P;
        for (int col0 = 0; col0 < ncol; col0 += cpp) {
            const int cl = tid % cpp, part = tid / cpp, col = col0 + cl;
            const bool active = part < P && col < ncol;
            const int r_lo = min(nb, part * run), r_hi = min(nb, r_lo + run);
            int sum = 0;
            if (active)
                for (int r = r_lo; r < r_hi; ++r) sum += stage[r * ncol + col];
            s_part[tid] = active ? sum : 0;
            __syncthreads();
            int running = 0;
            if (active) {
                running = s_tot[col];
                for (int p2 = 0; p2 < part; ++p2) running += s_part[p2 * cpp + cl];
                int* base = col < NC ? bc_base + col : bg_base + (col - NC);
                const int stride = col < NC ? NC : K;
                for (int r = r_lo; r < r_hi; ++r) {
                    base[(size_t)(b0 + r) * stride] = running;
                    running += stage[r * ncol + col];
                }
            }
            __syncthreads();                    // every reader of s_tot[col] and s_part is done
            if (active && part == P - 1) s_tot[col] = running;
        }
    }
    __syncthreads();
    for (int c = tid; c < ncol; c += NTHREADS) {    // totals in row nblk
        if (c < NC) bc_base[(size_t)nblk * NC + c] = s_tot[c];
        else bg_base[(size_t)nblk * K + (c - NC)] = s_tot[c];
    }

    int* cc = (int*)(ws + (is_query ? L.off_qcc : L.off_kcc)) + (size_t)bh * NC;
    int* co = (int*)(ws + (is_query ? L.off_qco : L.off_kco)) + (size_t)bh * (NC + 1);
    int* gc = (int*)(ws + (is_query ? L.off_qgc : L.off_kgc)) + (size_t)bh * K;
    int* go = (int*)(ws + (is_query ? L.off_qgo : L.off_kgo)) + (size_t)bh * (K + 1);
    const int pad = is_query ? L.BQ : KT;
    for (int c = tid; c < NC; c += NTHREADS) {
        const int v = s_tot[c];
        s_nt[c] = (v + L.BQ - 1) / L.BQ;
        cc[c] = v;
    }
    if (tid < K) gc[tid] = s_tot[NC + tid];
    __syncthreads();
    if (tid == 0) {
        int off = 0, tot = 0;
        for (int c = 0; c < NC; ++c) {
            co[c] = off;
            off += (s_tot[c] + pad - 1) / pad * pad;
            tot += s_nt[c];
        }
        co[NC] = off;
        *s_total = tot;
        int goff = 0;
        for (int g = 0; g < K; ++g) { go[g] = goff; goff += s_tot[NC + g]; }
        go[K] = goff;
    }
    // class -> group mask (written once, by the first query head)
    if (is_query && bh == 0) {
        uint32_t* clsmask = (uint32_t*)(ws + L.off_clsmask);
        for (int c = tid; c < NC; c += NTHREADS) {
            uint32_t m = 0;
            if (L.dense) {
                m = 0xffffffffu;
            } else {
                // exact classes: topk-subsets of the K groups in colex order; coarse classes: sets of
                // 1..topk of the S super-groups, by size, then colex
                uint32_t r = (uint32_t)c;
                int size = L.topk, top = K - 1;
                if (L.coarse) {
                    size = 1;
                    while (r >= binom_u32(L.S, size)) { r -= binom_u32(L.S, size); ++size; }
                    top = L.S - 1;
                }
                int g = top;
                for (int j = size; j >= 1; --j) {
                    while (binom_u32(g, j) > r) --g;      // largest g with C(g,j) <= r
                    m |= (1u << g);
                    r -= binom_u32(g, j);
                    --g;
                }
            }
            clsmask[c] = m;
        }
    }
    __syncthreads();
    if (!is_query) return;
    // Job list = the order in which the work-groups of the attention launch are dispatched.
    //  * Long sequences (256-row tiles, n >= LONG_N: a head's K and V no longer sit in the L2 of its XCD), class-major:
    //    the tiles of class 0 from its last (longest key walk) to its first, then class 1, ...  The work-groups
    //    resident at any moment are then neighbouring tiles of ONE class: they walk the same key classes from the
    //    same first tile at the same pace and share every K/V tile they fetch (at 1M tokens 1 TB is fetched from
    //    memory per launch instead of 20 TB).  The list still ends with short tiles, as the tail of the launch needs.
    //  * Otherwise slot-major: slot s = how many tiles from the end of its class a tile is; every class's last
    //    (longest-prefix) tile first.  K and V mostly stay in L2 at these lengths, and the mix of classes among the
    //    resident work-groups keeps them from asking for the same lines in the same cycles (class-major measured
    //    6 to 10 % slower at 131072 tokens with 8 groups).
    int* jobs = (int*)(ws + L.off_jobs) + (size_t)bh * L.NT;
    const int total = *s_total;
    for (int j = total + tid; j < L.NT; j += NTHREADS) jobs[j] = -1;
    for (int u = tid; u < total; u += NTHREADS) {                 // one thread per tile, tiles counted class by class
        int c = 0, first = 0;
        while (u >= first + s_nt[c]) { first += s_nt[c]; ++c; }
        const int ntc = s_nt[c], t = u - first;
        const int s = ntc - 1 - t;
        int j = first + s;
        if (!L.class_major) {
            j = 0;
            for (int c2 = 0; c2 < NC; ++c2) {
                j += min(s_nt[c2], s);
                if (c2 < c && s_nt[c2] > s) ++j;
            }
        }
        jobs[j] = (int)(((unsigned)c << 24) | (unsigned)t);       // t < 2^17: never the unused marker -1
    }
    __syncthreads();                                              // tmp may be reused by the caller
}

// scan + plan as a launch of its own (memberships given per token): one work-group per row
__global__ __launch_bounds__(SCAN_THREADS) void scan_plan_kernel(Layout L, char* __restrict__ ws)
{
    __shared__ int s_tmp[SCAN_PLAN_TMP_INTS];
    const int is_query = side_of_row(L, -1, blockIdx.x);
    const int bh = row_in_side(L, -1, blockIdx.x);
    scan_and_plan_row<SCAN_THREADS>(L, is_query, bh, ws, s_tmp, SCAN_PLAN_TMP_INTS);
}

template <typename T, int KMAX>
__global__ __launch_bounds__(SB) void score_topk_kernel(Layout L, HeadMap hm, const T* __restrict__ xq,
                                                        const T* __restrict__ xk,
                                                        const double* __restrict__ cent64, int which, int nbw,
                                                        char* __restrict__ ws)
{
    __shared__ __align__(16) char s_rows[SB * ROW_STRIDE];
    __shared__ int s_hist_c[MAX_CLASSES];
    __shared__ int s_hist_g[32];

    const int tid = threadIdx.x;
    const int blk0 = blockIdx.x * nbw;          // nbw consecutive sort blocks per work-group
    const int is_query = side_of_row(L, which, blockIdx.y);
    const int bh = row_in_side(L, which, blockIdx.y);
    const T* x = is_query ? xq : xk;
    const int H = is_query ? L.Hq : L.Hkv;
    const int h = bh % H;
    const int hk = is_query ? hm.kv[h] : h;
    const int d = L.d, K = L.K, n = L.n;
    constexpr int EPC = 16 / sizeof(T);                              // elements per 16-byte chunk
    constexpr int CPR = ROW_CHUNK_BYTES / 16;                        // chunks per staged row = loads per thread
    const int row_bytes = d * (int)sizeof(T);
    const int phases = (row_bytes + ROW_CHUNK_BYTES - 1) / ROW_CHUNK_BYTES;   // the last one may be partly past the row
    const int dcent = phases * (ROW_CHUNK_BYTES / (int)sizeof(T));              // rows of the (zero-padded) centroid table
    const int nb_here = min(nbw, L.nblk - blk0);
    const int total_steps = nb_here * phases;                        // (block, 128-byte column phase) pairs

    // centroids of this KV head as fp64 [d][KMAX]: a wave-uniform, read-only table -> scalar loads,
    // the values feed v_fma_f64 straight from SGPRs
    const double* __restrict__ cd = cent64 + (size_t)hk * dcent * KMAX;
    for (int e = tid; e < MAX_CLASSES; e += SB) s_hist_c[e] = 0;
    if (tid < 32) s_hist_g[tid] = 0;
    __syncthreads();                                                 // (the steps below have no barrier of their own)

    double acc[KMAX];
#pragma unroll
    for (int g = 0; g < KMAX; ++g) acc[g] = 0.0;

    uint32_t* masks = (uint32_t*)(ws + (is_query ? L.off_mq : L.off_mk));
    uint8_t* clsarr = (uint8_t*)(ws + (is_query ? L.off_qcls : L.off_kcls));
    const size_t cls_stride = is_query ? (size_t)n : (size_t)L.nblk * SB;
    // rows are row_bytes long; where they start comes from the strides of q (or of k)
    const long long* xs = is_query ? L.qs : L.ks;
    const size_t row_pitch = (size_t)xs[2] * sizeof(T);
    const char* xbase = (const char*)x + ((size_t)(bh / H) * xs[0] + (size_t)h * xs[1]) * sizeof(T);

    // Register staging of the next step: its global loads fly while the current step is computed.
    // Coalesced: consecutive threads fetch consecutive 16-byte chunks of a 128-byte row segment.
    u32x4 st[CPR];
#define FOCUS_SCORE_LOAD(STEP)                                                                       \
    do {                                                                                             \
        const int bi_ = (STEP) / phases, ph_ = (STEP) % phases;                                      \
        const int rows_ = min(SB, n - (blk0 + bi_) * SB);                                            \
        const char* g_ = xbase + (size_t)(blk0 + bi_) * SB * row_pitch + ph_ * ROW_CHUNK_BYTES;      \
        _Pragma("unroll") for (int i = 0; i < CPR; ++i) {                                            \
            const int cid_ = (tid & ~63) * CPR + i * 64 + (tid & 63);   /* chunk of this wavefront's 64 rows */ \
            const int r_ = cid_ / CPR, cc_ = cid_ % CPR;                                             \
            const u32x4 z_ = {0u, 0u, 0u, 0u};                                                       \
            const bool in_ = r_ < rows_ && ph_ * ROW_CHUNK_BYTES + cc_ * 16 < row_bytes;                 \
            st[i] = in_ ? *(const u32x4*)(g_ + (size_t)r_ * row_pitch + cc_ * 16) : z_;              \
        }                                                                                            \
    } while (0)

    FOCUS_SCORE_LOAD(0);
    for (int step = 0; step < total_steps; ++step) {
        const int bi = step / phases, ph = step % phases;
        // Every wavefront stages and reads its own 64 rows: LDS executes a wavefront's accesses in order, so no
        // barrier is needed, only the compiler must keep the order.
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int i = 0; i < CPR; ++i) {
            const int cid = (tid & ~63) * CPR + i * 64 + (tid & 63);
            *(u32x4*)(s_rows + (cid / CPR) * ROW_STRIDE + (cid % CPR) * 16) = st[i];
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        if (step + 1 < total_steps) FOCUS_SCORE_LOAD(step + 1);
        const int tbase = ph * (ROW_CHUNK_BYTES / (int)sizeof(T));
#pragma unroll 1
        for (int cc = 0; cc < CPR; ++cc) {
            const u32x4 val = *(const u32x4*)(s_rows + tid * ROW_STRIDE + cc * 16);
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
                    xv[2 * e] = (double)bf16_bits_to_f32((uint16_t)(val[e] & 0xffffu));
                    xv[2 * e + 1] = (double)bf16_bits_to_f32((uint16_t)(val[e] >> 16));
                }
            }
#pragma unroll
            for (int e = 0; e < EPC; ++e) {
                const double* cr = cd + (size_t)(tbase + cc * EPC + e) * KMAX;
#pragma unroll
                for (int g = 0; g < KMAX; ++g) acc[g] = fma(xv[e], cr[g], acc[g]);
            }
        }
        if (ph != phases - 1) continue;

        // ---- a sort block is complete: top-k by rank counting; ties go to the smaller group index
        const int blk = blk0 + bi;
        const int pos = blk * SB + tid;
        uint32_t mask = 0;
#pragma unroll
        for (int g = 0; g < KMAX; ++g) {
            if (g < K) {
                int beaten = 0;
#pragma unroll
                for (int o = 0; o < KMAX; ++o) {
                    if (o < K && o != g)
                        beaten += (acc[o] > acc[g] || (acc[o] == acc[g] && o < g)) ? 1 : 0;
                }
                if (beaten < L.topk) mask |= (1u << g);
            }
        }
        // A NaN score loses no comparison and would add its group to the topk others: a membership that is not
        // a topk-subset has no class.  Such a token (only a NaN can cause it) takes the first topk groups.
        if (__popc(mask) != L.topk) mask = (L.topk == 32) ? 0xffffffffu : ((1u << L.topk) - 1u);
#pragma unroll
        for (int g = 0; g < KMAX; ++g) acc[g] = 0.0;
        // class = colex rank of the membership set among all topk-subsets
        int cls = 0;
        if (L.coarse) {
            cls = class_of_mask(mask, 0, 1, L.S);
        } else if (!L.dense) {
            int j = 0;
            for (int g = 0; g < K; ++g)
                if ((mask >> g) & 1u) { ++j; cls += (int)g_binom.v[g * 33 + j]; }
        }
        if (pos < n) {
            masks[(size_t)bh * n + pos] = mask;
            clsarr[(size_t)bh * cls_stride + pos] = (uint8_t)cls;
            atomicAdd(&s_hist_c[cls], 1);
            for (int g = 0; g < K; ++g)
                if ((mask >> g) & 1u) atomicAdd(&s_hist_g[g], 1);
        }
        __syncthreads();
        int* bc = (int*)(ws + (is_query ? L.off_qbc : L.off_kbc)) + ((size_t)bh * (L.nblk + 1) + blk) * L.NC;
        int* bg = (int*)(ws + (is_query ? L.off_qbg : L.off_kbg)) + ((size_t)bh * (L.nblk + 1) + blk) * K;
        for (int c = tid; c < L.NC; c += SB) { bc[c] = s_hist_c[c]; s_hist_c[c] = 0; }
        if (tid < K) { bg[tid] = s_hist_g[tid]; s_hist_g[tid] = 0; }
        __syncthreads();                                             // cleared before the next block's atomics
    }
#undef FOCUS_SCORE_LOAD
}

// ---------------------------------------------------------------- start of an assign pass
// The largest-key-norm slots to zero and, when centroids are given, their fp64 table: one small launch.
__global__ __launch_bounds__(256) void assign_init_kernel(unsigned* __restrict__ zeros, size_t nzeros,
                                                          const float* __restrict__ cents,
                                                          double* __restrict__ cent64, int Hkv, int K, int d, int dcent, int kmax)
{
    const size_t step = (size_t)gridDim.x * blockDim.x;
    const size_t i0 = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    for (size_t i = i0; i < nzeros; i += step) zeros[i] = 0u;
    if (cents) {
        const size_t total = (size_t)Hkv * dcent * kmax;
        for (size_t e = i0; e < total; e += step) {
            const int g = (int)(e % kmax), t = (int)((e / kmax) % dcent), hk = (int)(e / ((size_t)kmax * dcent));
            cent64[e] = (g < K && t < d) ? (double)cents[((size_t)hk * K + g) * d + t] : 0.0;
        }
    }
}

__global__ void fill_i32_kernel(int* __restrict__ p, size_t count, int value)
{
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t step = (size_t)gridDim.x * blockDim.x;
    for (; i < count; i += step) p[i] = value;
}

// ---------------------------------------------------------------- scatter
// sum of the squares of the eight 16-bit values of a chunk (bf16 or IEEE half bit patterns)
__device__ inline float chunk_norm2(const uint4& val, bool f16)
{
    const uint32_t w[4] = {val.x, val.y, val.z, val.w};
    float acc = 0.f;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const float a = f16 ? f16_bits_to_f32((uint16_t)(w[e] & 0xffffu)) : __uint_as_float(w[e] << 16);
        const float b = f16 ? f16_bits_to_f32((uint16_t)(w[e] >> 16)) : __uint_as_float(w[e] & 0xffff0000u);
        acc = fmaf(a, a, acc);
        acc = fmaf(b, b, acc);
    }
    return acc;
}

// k: the key rows (16-bit types) for the class-ordered copy the matrix-core attention kernel reads, or NULL.
// The copy also leaves the largest squared key norm of the (batch, KV head) in the workspace (off_kn2: KN2_SLOTS
// partial maxima per head, cleared by assign_init): a non-negative float orders like its bit pattern, so one
// atomicMax on the bits per work-group does it, and a NaN or infinite norm ends up above every finite one.
__global__ __launch_bounds__(SB) void scatter_kernel(Layout L, int which, const uint16_t* __restrict__ k, char* __restrict__ ws)
{
    __shared__ int s_wc[4][MAX_CLASSES];
    __shared__ int s_wg[4][32];
    __shared__ int s_dest[SB];
    __shared__ unsigned s_n2[SB / 64];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int blk = blockIdx.x;
    // the key rows (the long ones: they copy their sort block of K) are dispatched first
    const unsigned yrow = gridDim.y - 1u - blockIdx.y;
    const int is_query = side_of_row(L, which, yrow);
    const int bh = row_in_side(L, which, yrow);
    const int n = L.n, NC = L.NC, K = L.K;
    const int pos = blk * SB + tid;
    const bool valid = pos < n;
    const uint32_t* masks = (const uint32_t*)(ws + (is_query ? L.off_mq : L.off_mk));
    const uint8_t* clsarr = (const uint8_t*)(ws + (is_query ? L.off_qcls : L.off_kcls));
    const size_t cls_stride = is_query ? (size_t)n : (size_t)L.nblk * SB;
    const uint32_t mask = valid ? masks[(size_t)bh * n + pos] : 0u;
    const int cls = valid ? (int)clsarr[(size_t)bh * cls_stride + pos] : -1;

    for (int e = tid; e < 4 * MAX_CLASSES; e += SB) (&s_wc[0][0])[e] = 0;
    __syncthreads();

    const unsigned long long lt = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
    // stable rank among the tokens of the same class inside this wavefront
    int rank_c = 0;
    unsigned long long todo = __ballot(valid);
    while (todo) {
        const int leader = __ffsll((long long)todo) - 1;
        const int c0 = __shfl(cls, leader, 64);
        const unsigned long long same = __ballot(valid && cls == c0);
        if (valid && cls == c0) rank_c = __popcll(same & lt);
        if (lane == leader) s_wc[wave][c0] = __popcll(same);
        todo &= ~same;
    }
    // per-wavefront totals of every group bit
    for (int g = 0; g < K; ++g) {
        const unsigned long long has = __ballot(valid && ((mask >> g) & 1u));
        if (lane == 0) s_wg[wave][g] = __popcll(has);
    }
    __syncthreads();

    const int* bc = (const int*)(ws + (is_query ? L.off_qbc : L.off_kbc)) + ((size_t)bh * (L.nblk + 1) + blk) * NC;
    const int* bg = (const int*)(ws + (is_query ? L.off_qbg : L.off_kbg)) + ((size_t)bh * (L.nblk + 1) + blk) * K;
    const int* co = (const int*)(ws + (is_query ? L.off_qco : L.off_kco)) + (size_t)bh * (NC + 1);
    const int* go = (const int*)(ws + (is_query ? L.off_qgo : L.off_kgo)) + (size_t)bh * (K + 1);
    int dest = -1;
    if (valid) {
        int before = 0;
        for (int w = 0; w < wave; ++w) before += s_wc[w][cls];
        dest = co[cls] + bc[cls] + before + rank_c;
        if (is_query) {
            ((int*)(ws + L.off_qperm))[(size_t)bh * L.NQP + dest] = pos;
        } else {
            ((int*)(ws + L.off_kpos))[(size_t)bh * L.NKP + dest] = pos;
            if (L.coarse) ((uint32_t*)(ws + L.off_kmsk))[(size_t)bh * L.NKP + dest] = mask;
        }
    }
    // group lists: position-ascending because ranks follow the position order
    int* lists = (int*)(ws + (is_query ? L.off_qgl : L.off_kgl)) + (size_t)bh * L.topk * n;
    for (int g = 0; g < K; ++g) {
        const bool mine = valid && ((mask >> g) & 1u);
        const unsigned long long has = __ballot(mine);
        if (mine) {
            int bw = 0;
            for (int w = 0; w < wave; ++w) bw += s_wg[w][g];
            lists[go[g] + bg[g] + bw + __popcll(has & lt)] = pos;
        }
    }

    // ---- pads of the class-ordered arrays: the work-group of sort block b fills those of the classes b, b + nblk, ...
    // (class NC stands for the unused end of the arrays).  qperm -1, kpos KPOS_PAD, masks and key rows zero.
    const int* cnt = (const int*)(ws + (is_query ? L.off_qcc : L.off_kcc)) + (size_t)bh * NC;
    const int plen = is_query ? L.NQP : L.NKP;
    const bool copy_k = !is_query && k != nullptr;
    const int CPR = L.dp / 8;                        // 16-byte chunks per row of the key copy (8, 16 or 32)
    uint4* kc = (uint4*)(ws + L.off_kc) + (size_t)bh * L.NKP * CPR;
    for (int c = blk; c <= NC; c += L.nblk) {
        const int p0 = c < NC ? co[c] + cnt[c] : co[NC];
        const int p1 = c < NC ? co[c + 1] : plen;
        for (int p = p0 + tid; p < p1; p += SB) {
            if (is_query) {
                ((int*)(ws + L.off_qperm))[(size_t)bh * L.NQP + p] = -1;
            } else {
                ((int*)(ws + L.off_kpos))[(size_t)bh * L.NKP + p] = KPOS_PAD;
                if (L.coarse) ((uint32_t*)(ws + L.off_kmsk))[(size_t)bh * L.NKP + p] = 0u;
            }
        }
        if (copy_k && c < NC)                        // (nothing reads the key rows past the last class)
            for (int id = tid; id < (p1 - p0) * CPR; id += SB) kc[(size_t)p0 * CPR + id] = make_uint4(0, 0, 0, 0);
    }

    // ---- key rows: this sort block's rows into their class-ordered places, d padded with zeros to dp
    if (!copy_k) return;
    s_dest[tid] = dest;
    __syncthreads();
    const int cin = L.d / 8;                         // chunks of a source row
    const bool f16 = L.dtype == 2;
    // source rows through the strides of k (multiples of 8 elements = one 16-byte chunk)
    const uint4* src = (const uint4*)k + ((size_t)(bh / L.Hkv) * L.ks[0] + (size_t)(bh % L.Hkv) * L.ks[1] + (size_t)blk * SB * L.ks[2]) / 8;
    const size_t pitch = (size_t)L.ks[2] / 8;
    unsigned n2max = 0u;
    for (int id = tid; id < SB * CPR; id += SB) {
        const int row = id / CPR, ch = id % CPR;
        const int dd = s_dest[row];
        uint4 val = make_uint4(0, 0, 0, 0);
        if (dd >= 0) {
            if (ch < cin) val = src[(size_t)row * pitch + ch];
            kc[(size_t)dd * CPR + ch] = val;
        }
        // the CPR chunks of a row sit in CPR consecutive lanes (CPR a power of two <= 32, rows do not straddle waves)
        float n2 = chunk_norm2(val, f16);
        for (int off = 1; off < CPR; off <<= 1) n2 += __shfl_xor(n2, off, 64);
        const unsigned bits = __float_as_uint(n2) & 0x7fffffffu;     // a NaN may carry a sign bit
        n2max = bits > n2max ? bits : n2max;
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        const unsigned o = (unsigned)__shfl_xor((int)n2max, off, 64);
        n2max = o > n2max ? o : n2max;
    }
    if (lane == 0) s_n2[wave] = n2max;
    __syncthreads();
    if (tid == 0) {
        for (int w = 1; w < SB / 64; ++w) n2max = s_n2[w] > n2max ? s_n2[w] : n2max;
        // KN2_SLOTS slots per head, so that the work-groups of a head do not queue up on one address
        if (n2max != 0u) atomicMax((unsigned*)(ws + L.off_kn2) + (size_t)bh * KN2_SLOTS + (blk % KN2_SLOTS), n2max);
    }
}

// ---------------------------------------------------------------- membership given per token
// The paper's router assigns one membership per token of a layer, shared by all heads and by the
// query and key roles (Sec. 2).  One work-group per (sort block, batch element) turns the token
// masks into class ids and histograms once and writes them for every query and KV head, in the
// same places score_topk fills.  A mask that is not a topk-subset of the K groups would index
// outside the class tables: it is replaced by the first topk groups and counted.
__global__ __launch_bounds__(SB) void token_classes_kernel(Layout L, const uint32_t* __restrict__ token_masks,
                                                           char* __restrict__ ws, int32_t* __restrict__ invalid_count)
{
    __shared__ int s_hist_c[MAX_CLASSES];
    __shared__ int s_hist_g[32];
    const int tid = threadIdx.x;
    const int blk = blockIdx.x, b = blockIdx.y;
    const int n = L.n, K = L.K;
    const int pos = blk * SB + tid;
    for (int e = tid; e < MAX_CLASSES; e += SB) s_hist_c[e] = 0;
    if (tid < 32) s_hist_g[tid] = 0;
    __syncthreads();
    uint32_t mask = 0;
    int cls = 0;
    if (pos < n) {
        // no masks given: every token in the first topk groups (callers that need one class in position order)
        mask = token_masks ? token_masks[(size_t)b * n + pos] : ((L.topk == 32) ? 0xffffffffu : ((1u << L.topk) - 1u));
        const uint32_t allowed = (K == 32) ? 0xffffffffu : ((1u << K) - 1u);
        if ((mask & ~allowed) != 0u || __popc(mask) != L.topk) {
            mask = (L.topk == 32) ? 0xffffffffu : ((1u << L.topk) - 1u);
            if (invalid_count) atomicAdd(invalid_count, 1);
        }
        if (L.coarse) {
            cls = class_of_mask(mask, 0, 1, L.S);
        } else if (!L.dense) {
            int j = 0;
            for (int g = 0; g < K; ++g)
                if ((mask >> g) & 1u) { ++j; cls += (int)g_binom.v[g * 33 + j]; }
        }
        atomicAdd(&s_hist_c[cls], 1);
        for (int g = 0; g < K; ++g)
            if ((mask >> g) & 1u) atomicAdd(&s_hist_g[g], 1);
    }
    __syncthreads();
    for (int is_query = 1; is_query >= 0; --is_query) {
        const int H = is_query ? L.Hq : L.Hkv;
        uint32_t* masks = (uint32_t*)(ws + (is_query ? L.off_mq : L.off_mk));
        uint8_t* clsarr = (uint8_t*)(ws + (is_query ? L.off_qcls : L.off_kcls));
        const size_t cls_stride = is_query ? (size_t)n : (size_t)L.nblk * SB;
        for (int h = 0; h < H; ++h) {
            const size_t bh = (size_t)b * H + h;
            if (pos < n) {
                masks[bh * n + pos] = mask;
                clsarr[bh * cls_stride + pos] = (uint8_t)cls;
            }
            int* bc = (int*)(ws + (is_query ? L.off_qbc : L.off_kbc)) + (bh * (L.nblk + 1) + blk) * L.NC;
            int* bg = (int*)(ws + (is_query ? L.off_qbg : L.off_kbg)) + (bh * (L.nblk + 1) + blk) * K;
            for (int c = tid; c < L.NC; c += SB) bc[c] = s_hist_c[c];
            if (tid < K) bg[tid] = s_hist_g[tid];
        }
    }
}

// Sort blocks per work-group of the scoring launch: up to four (a work-group prefetches its next block while it
// computes), fewer when that would leave the chip with less than a few work-groups per slot to balance with.
int score_blocks_per_group(long long items)
{
    const long long slots = 256 * 4;
    int nbw = 4;
    while (nbw > 1 && items / nbw < 4 * slots) nbw >>= 1;
    return nbw;
}

// scores and memberships of the queries and of the keys, one launch: query rows first, key rows after them
template <typename T>
hipError_t launch_score(const Layout& L, const HeadMap& hm, const void* q, const void* k, char* ws, hipStream_t st)
{
    const int kmax = L.K <= 4 ? 4 : L.K <= 8 ? 8 : L.K <= 16 ? 16 : 32;
    const double* cent64 = (const double*)(ws + L.off_cent64);
    // (more rows than one launch can have: the two sides one after the other)
    const bool both = L.B * (L.Hq + L.Hkv) <= MAX_GRID_ROWS;
    for (int which = both ? -1 : 1; which >= -1; --which) {
        const int rows = which < 0 ? L.B * (L.Hq + L.Hkv) : which ? L.B * L.Hq : L.B * L.Hkv;
        const int nbw = score_blocks_per_group((long long)rows * L.nblk);
        dim3 grid((L.nblk + nbw - 1) / nbw, rows);
#define FOCUS_SCORE(KM_) hipLaunchKernelGGL((score_topk_kernel<T, KM_>), grid, dim3(SB), 0, st, L, hm, (const T*)q, (const T*)k, cent64, which, nbw, ws)
        switch (kmax) {
            case 4: FOCUS_SCORE(4); break;
            case 8: FOCUS_SCORE(8); break;
            case 16: FOCUS_SCORE(16); break;
            default: FOCUS_SCORE(32); break;
        }
#undef FOCUS_SCORE
        if (which <= 0) break;
    }
    return hipGetLastError();
}

}  // namespace

namespace {

// the key-norm slots to zero and, with centroids given, their fp64 table [Hkv][dcent][kmax]
void launch_assign_init(const Layout& L, const float* centroids, char* ws, hipStream_t st)
{
    const size_t nzeros = (size_t)L.B * L.Hkv * KN2_SLOTS;           // the largest-key-norm slots
    const int kmax = L.K <= 4 ? 4 : L.K <= 8 ? 8 : L.K <= 16 ? 16 : 32;
    const int row_bytes = L.d * L.elem;
    const int dcent = (row_bytes + ROW_CHUNK_BYTES - 1) / ROW_CHUNK_BYTES * (ROW_CHUNK_BYTES / L.elem);
    const size_t work = std::max(nzeros, centroids ? (size_t)L.Hkv * dcent * kmax : (size_t)0);
    const int grid = (int)std::min((size_t)1024, (work + 255) / 256);
    hipLaunchKernelGGL(assign_init_kernel, dim3(grid), dim3(256), 0, st, (unsigned*)(ws + L.off_kn2), nzeros,
                       centroids, (double*)(ws + L.off_cent64), L.Hkv, L.K, L.d, dcent, kmax);
}

// from class ids, block prefixes and the per-row plan to the class-ordered arrays, group lists and key copy
hipError_t launch_scatter(const Layout& L, const void* k, char* ws, hipStream_t st)
{
    // query side and key side in the same launch: rows [0, B*Hq) and the B*Hkv rows after them
    // (more rows than one launch can have: the two sides one after the other)
    const uint16_t* kcopy = L.dtype != 0 ? (const uint16_t*)k : nullptr;   // class-ordered key copy for the MFMA kernel
    const bool both = L.B * (L.Hq + L.Hkv) <= MAX_GRID_ROWS;
    for (int which = both ? -1 : 1; which >= -1; --which) {
        const int rows = which < 0 ? L.B * (L.Hq + L.Hkv) : which ? L.B * L.Hq : L.B * L.Hkv;
        hipLaunchKernelGGL(scatter_kernel, dim3(L.nblk, rows), dim3(SB), 0, st, L, which, kcopy, ws);
        if (which <= 0) break;
    }
    return hipGetLastError();
}

}  // namespace

hipError_t launch_assign(const Layout& L, const HeadMap& hm, const void* q, const void* k,
                         const float* centroids, char* ws, hipStream_t st)
{
    hipError_t e;
    launch_assign_init(L, centroids, ws, st);
    if (L.dtype == 0) e = launch_score<float>(L, hm, q, k, ws, st);
    else if (L.dtype == 2) e = launch_score<f16_bits>(L, hm, q, k, ws, st);
    else e = launch_score<uint16_t>(L, hm, q, k, ws, st);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(scan_plan_kernel, dim3(L.B * (L.Hq + L.Hkv)), dim3(SCAN_THREADS), 0, st, L, ws);
    return launch_scatter(L, k, ws, st);
}

hipError_t launch_assign_tokens(const Layout& L, const uint32_t* token_masks, const void* k, char* ws,
                                int32_t* invalid_count, hipStream_t st)
{
    launch_assign_init(L, nullptr, ws, st);
    if (invalid_count) hipLaunchKernelGGL(fill_i32_kernel, dim3(1), dim3(64), 0, st, invalid_count, (size_t)1, 0);
    hipLaunchKernelGGL(token_classes_kernel, dim3(L.nblk, L.B), dim3(SB), 0, st, L, token_masks, ws, invalid_count);
    hipLaunchKernelGGL(scan_plan_kernel, dim3(L.B * (L.Hq + L.Hkv)), dim3(SCAN_THREADS), 0, st, L, ws);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    return launch_scatter(L, k, ws, st);
}

}  // namespace focus
