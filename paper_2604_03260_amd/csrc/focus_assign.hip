// focus_assign: centroid scoring, top-k membership, bucketing by group and by
// membership class (Sec. 2 Eq. 1 in per-head dot-product form; Sec. 2
// "Efficiency at inference"; the stable sort by group of App. D done as a
// counting sort).
//
// Kernels, all launched per (sort block of SB positions, batch*head):
//   score_topk   streams q (or k) once, scores every token against the K
//                centroids of its KV head in fp64 (products are exact in fp64,
//                added in index order, so the result is reproducible bit for
//                bit), keeps the top-k groups, writes the membership mask, the
//                class id and the per-block histograms of classes and groups;
//   scan_blocks  exclusive scan of the histograms over the sort blocks;
//   plan_heads   class offsets (padded to tile multiples), group list offsets,
//                the class -> group-mask table and the heaviest-first job list
//                of query tiles;
//   scatter      stable ranks inside a block by wavefront ballot + popcount,
//                coalesced 4-byte writes of the class-ordered position arrays
//                and of the per-group index lists.
#include "focus_internal.h"
#include <hip/hip_bf16.h>
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

constexpr int NBW = 4;          // sort blocks handled by one work-group of the scoring kernel

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// The kernels of the bucketing serve the query side, the key side, or both in one launch (which = 1, 0, -1):
// with both, the rows [0, B*Hq) of the launch are query (batch, head) pairs and the B*Hkv after them key pairs.
constexpr int MAX_GRID_ROWS = 65535;
__device__ inline int side_of_row(const Layout& L, int which, unsigned row) { return which < 0 ? (int)(row < (unsigned)(L.B * L.Hq)) : which; }
__device__ inline int row_in_side(const Layout& L, int which, unsigned row)
{
    return (which < 0 && row >= (unsigned)(L.B * L.Hq)) ? (int)row - L.B * L.Hq : (int)row;
}

template <typename T, int KMAX>
__global__ __launch_bounds__(SB) void score_topk_kernel(Layout L, HeadMap hm, const T* __restrict__ xq,
                                                        const T* __restrict__ xk,
                                                        const double* __restrict__ cent64, int which,
                                                        char* __restrict__ ws)
{
    __shared__ __align__(16) char s_rows[SB * ROW_STRIDE];
    __shared__ int s_hist_c[MAX_CLASSES];
    __shared__ int s_hist_g[32];

    const int tid = threadIdx.x;
    const int blk0 = blockIdx.x * NBW;
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
    const int nb_here = min(NBW, L.nblk - blk0);
    const int total_steps = nb_here * phases;                        // (block, 128-byte column phase) pairs

    // centroids of this KV head as fp64 [d][KMAX]: a wave-uniform, read-only table -> scalar loads,
    // the values feed v_fma_f64 straight from SGPRs
    const double* __restrict__ cd = cent64 + (size_t)hk * dcent * KMAX;
    for (int e = tid; e < MAX_CLASSES; e += SB) s_hist_c[e] = 0;
    if (tid < 32) s_hist_g[tid] = 0;

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
            const int cid_ = tid + i * SB;                                                           \
            const int r_ = cid_ / CPR, cc_ = cid_ % CPR;                                             \
            const u32x4 z_ = {0u, 0u, 0u, 0u};                                                       \
            const bool in_ = r_ < rows_ && ph_ * ROW_CHUNK_BYTES + cc_ * 16 < row_bytes;                 \
            st[i] = in_ ? *(const u32x4*)(g_ + (size_t)r_ * row_pitch + cc_ * 16) : z_;              \
        }                                                                                            \
    } while (0)

    FOCUS_SCORE_LOAD(0);
    for (int step = 0; step < total_steps; ++step) {
        const int bi = step / phases, ph = step % phases;
        __syncthreads();                                             // the previous step's reads are done
#pragma unroll
        for (int i = 0; i < CPR; ++i) {
            const int cid = tid + i * SB;
            *(u32x4*)(s_rows + (cid / CPR) * ROW_STRIDE + (cid % CPR) * 16) = st[i];
        }
        __syncthreads();
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
        // the next block's atomics come after the two barriers of its first step
    }
#undef FOCUS_SCORE_LOAD
}

// ---------------------------------------------------------------- scans over sort blocks
// One work-group per (column, batch*head): exclusive scan of a histogram column
// over the sort blocks, total in row nblk.
__global__ __launch_bounds__(256) void scan_blocks_kernel(Layout L, int which, char* __restrict__ ws)
{
    __shared__ int s_wave[4];
    __shared__ int s_carry;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int col = blockIdx.x;           // [0,NC): class column, [NC,NC+K): group column
    const int is_query = side_of_row(L, which, blockIdx.y);
    const int bh = row_in_side(L, which, blockIdx.y);
    int* base;
    int stride;
    if (col < L.NC) {
        base = (int*)(ws + (is_query ? L.off_qbc : L.off_kbc)) + (size_t)bh * (L.nblk + 1) * L.NC + col;
        stride = L.NC;
    } else {
        base = (int*)(ws + (is_query ? L.off_qbg : L.off_kbg)) + (size_t)bh * (L.nblk + 1) * L.K + (col - L.NC);
        stride = L.K;
    }
    if (tid == 0) s_carry = 0;
    __syncthreads();
    for (int b0 = 0; b0 < L.nblk; b0 += 256) {
        const int b = b0 + tid;
        const int v = (b < L.nblk) ? base[(size_t)b * stride] : 0;
        int incl = v;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            int o = __shfl_up(incl, off, 64);
            if (lane >= off) incl += o;
        }
        if (lane == 63) s_wave[wave] = incl;
        __syncthreads();
        int wbase = 0;
        for (int w = 0; w < wave; ++w) wbase += s_wave[w];
        const int carry = s_carry;
        if (b < L.nblk) base[(size_t)b * stride] = carry + wbase + incl - v;
        __syncthreads();
        if (tid == 255) s_carry = carry + wbase + incl;
        __syncthreads();
    }
    if (tid == 0) base[(size_t)L.nblk * stride] = s_carry;
}

// ---------------------------------------------------------------- per-head plan
__global__ __launch_bounds__(256) void plan_heads_kernel(Layout L, int which, char* __restrict__ ws)
{
    __shared__ int s_cnt[MAX_CLASSES];
    __shared__ int s_nt[MAX_CLASSES];
    __shared__ int s_total;
    const int tid = threadIdx.x;
    const int is_query = side_of_row(L, which, blockIdx.x);
    const int bh = row_in_side(L, which, blockIdx.x);
    const int NC = L.NC, K = L.K;
    const int* bc_tot = (const int*)(ws + (is_query ? L.off_qbc : L.off_kbc)) + ((size_t)bh * (L.nblk + 1) + L.nblk) * NC;
    const int* bg_tot = (const int*)(ws + (is_query ? L.off_qbg : L.off_kbg)) + ((size_t)bh * (L.nblk + 1) + L.nblk) * K;
    int* cc = (int*)(ws + (is_query ? L.off_qcc : L.off_kcc)) + (size_t)bh * NC;
    int* co = (int*)(ws + (is_query ? L.off_qco : L.off_kco)) + (size_t)bh * (NC + 1);
    int* gc = (int*)(ws + (is_query ? L.off_qgc : L.off_kgc)) + (size_t)bh * K;
    int* go = (int*)(ws + (is_query ? L.off_qgo : L.off_kgo)) + (size_t)bh * (K + 1);
    const int pad = is_query ? L.BQ : KT;

    for (int c = tid; c < NC; c += 256) {
        int v = bc_tot[c];
        s_cnt[c] = v;
        s_nt[c] = (v + L.BQ - 1) / L.BQ;
        cc[c] = v;
    }
    if (tid < K) gc[tid] = bg_tot[tid];
    __syncthreads();
    if (tid == 0) {
        int off = 0, tot = 0;
        for (int c = 0; c < NC; ++c) {
            co[c] = off;
            off += (s_cnt[c] + pad - 1) / pad * pad;
            tot += s_nt[c];
        }
        co[NC] = off;
        s_total = tot;
        int goff = 0;
        for (int g = 0; g < K; ++g) { go[g] = goff; goff += bg_tot[g]; }
        go[K] = goff;
    }
    // class -> group mask (written once, by the first query head)
    if (is_query && bh == 0) {
        uint32_t* clsmask = (uint32_t*)(ws + L.off_clsmask);
        for (int c = tid; c < NC; c += 256) {
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
    const int total = s_total;
    for (int j = total + tid; j < L.NT; j += 256) jobs[j] = -1;
    int first = 0;
    for (int c = 0; c < NC; ++c) {
        const int ntc = s_nt[c];
        for (int t = tid; t < ntc; t += 256) {
            const int s = ntc - 1 - t;
            int j = first + s;
            if (!L.class_major) {
                j = 0;
                for (int c2 = 0; c2 < NC; ++c2) {
                    j += min(s_nt[c2], s);
                    if (c2 < c && s_nt[c2] > s) ++j;
                }
            }
            jobs[j] = (int)(((unsigned)c << 24) | (unsigned)t);   // t < 2^17: never the unused marker -1
        }
        first += ntc;
    }
}

// ---------------------------------------------------------------- start of an assign pass
// Pads of the class-ordered position arrays (qperm -1, kpos KPOS_PAD, the key masks of coarse classes 0), the
// largest-key-norm slots (0) and, when centroids are given, their fp64 table: one launch.
__global__ __launch_bounds__(256) void assign_init_kernel(int* __restrict__ qperm, size_t nq, int* __restrict__ kpos, size_t nk,
                                                          int* __restrict__ kmsk, unsigned* __restrict__ kn2, size_t nkn2,
                                                          const float* __restrict__ cents,
                                                          double* __restrict__ cent64, int Hkv, int K, int d, int dcent, int kmax)
{
    const size_t step = (size_t)gridDim.x * blockDim.x;
    const size_t i0 = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    for (size_t i = i0; i < nkn2; i += step) kn2[i] = 0u;
    for (size_t i = i0; i < nq; i += step) qperm[i] = -1;
    for (size_t i = i0; i < nk; i += step) kpos[i] = KPOS_PAD;
    if (kmsk)
        for (size_t i = i0; i < nk; i += step) kmsk[i] = 0;
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
__global__ __launch_bounds__(SB) void scatter_kernel(Layout L, int which, char* __restrict__ ws)
{
    __shared__ int s_wc[4][MAX_CLASSES];
    __shared__ int s_wg[4][32];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int blk = blockIdx.x;
    const int is_query = side_of_row(L, which, blockIdx.y);
    const int bh = row_in_side(L, which, blockIdx.y);
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
    if (valid) {
        int before = 0;
        for (int w = 0; w < wave; ++w) before += s_wc[w][cls];
        const int dest = co[cls] + bc[cls] + before + rank_c;
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

// scores and memberships of the queries and of the keys, one launch: query rows first, key rows after them
template <typename T>
hipError_t launch_score(const Layout& L, const HeadMap& hm, const void* q, const void* k, char* ws, hipStream_t st)
{
    const int kmax = L.K <= 4 ? 4 : L.K <= 8 ? 8 : L.K <= 16 ? 16 : 32;
    const double* cent64 = (const double*)(ws + L.off_cent64);
    // (more rows than one launch can have: the two sides one after the other)
    const bool both = L.B * (L.Hq + L.Hkv) <= MAX_GRID_ROWS;
    for (int which = both ? -1 : 1; which >= -1; --which) {
        dim3 grid((L.nblk + NBW - 1) / NBW, which < 0 ? L.B * (L.Hq + L.Hkv) : which ? L.B * L.Hq : L.B * L.Hkv);
#define FOCUS_SCORE(KM_) hipLaunchKernelGGL((score_topk_kernel<T, KM_>), grid, dim3(SB), 0, st, L, hm, (const T*)q, (const T*)k, cent64, which, ws)
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

// pads of the class-ordered position arrays and, with centroids given, their fp64 table [Hkv][dcent][kmax]
void launch_assign_init(const Layout& L, const float* centroids, char* ws, hipStream_t st)
{
    const size_t nq = (size_t)L.B * L.Hq * L.NQP, nk = (size_t)L.B * L.Hkv * L.NKP;
    const int grid = (int)min((size_t)8192, (max(nq, nk) + 255) / 256);
    const int kmax = L.K <= 4 ? 4 : L.K <= 8 ? 8 : L.K <= 16 ? 16 : 32;
    const int row_bytes = L.d * L.elem;
    const int dcent = (row_bytes + ROW_CHUNK_BYTES - 1) / ROW_CHUNK_BYTES * (ROW_CHUNK_BYTES / L.elem);
    hipLaunchKernelGGL(assign_init_kernel, dim3(grid), dim3(256), 0, st, (int*)(ws + L.off_qperm), nq, (int*)(ws + L.off_kpos), nk,
                       L.coarse ? (int*)(ws + L.off_kmsk) : nullptr, (unsigned*)(ws + L.off_kn2), (size_t)L.B * L.Hkv * KN2_SLOTS,
                       centroids, (double*)(ws + L.off_cent64), L.Hkv, L.K, L.d, dcent, kmax);
}

// from masks, class ids and block histograms to the class-ordered arrays, group lists and job lists
hipError_t launch_bucketing(const Layout& L, const void* k, char* ws, hipStream_t st)
{
    // query side and key side in the same launches: rows [0, B*Hq) and the B*Hkv rows after them
    // (more rows than one launch can have: the two sides one after the other)
    const bool both = L.B * (L.Hq + L.Hkv) <= MAX_GRID_ROWS;
    for (int which = both ? -1 : 1; which >= -1; --which) {
        const int rows = which < 0 ? L.B * (L.Hq + L.Hkv) : which ? L.B * L.Hq : L.B * L.Hkv;
        hipLaunchKernelGGL(scan_blocks_kernel, dim3(L.NC + L.K, rows), dim3(256), 0, st, L, which, ws);
        hipLaunchKernelGGL(plan_heads_kernel, dim3(rows), dim3(256), 0, st, L, which, ws);
        hipLaunchKernelGGL(scatter_kernel, dim3(L.nblk, rows), dim3(SB), 0, st, L, which, ws);
        if (which <= 0) break;
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (L.dtype != 0) return launch_gather_k(L, k, ws, st);   // class-ordered key copy for the MFMA kernel
    return hipSuccess;
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
    return launch_bucketing(L, k, ws, st);
}

hipError_t launch_assign_tokens(const Layout& L, const uint32_t* token_masks, const void* k, char* ws,
                                int32_t* invalid_count, hipStream_t st)
{
    launch_assign_init(L, nullptr, ws, st);
    if (invalid_count) hipLaunchKernelGGL(fill_i32_kernel, dim3(1), dim3(64), 0, st, invalid_count, (size_t)1, 0);
    hipLaunchKernelGGL(token_classes_kernel, dim3(L.nblk, L.B), dim3(SB), 0, st, L, token_masks, ws, invalid_count);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    return launch_bucketing(L, k, ws, st);
}

}  // namespace focus
