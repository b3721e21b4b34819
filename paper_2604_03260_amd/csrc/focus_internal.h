// Internal layout of the workspace and the launch entry points shared by the
// translation units of libfocus.so.  Not part of the public ABI.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

namespace focus {

constexpr int SB = 256;        // positions per sort block (one work-group of the bucketing kernels)
constexpr int BQ_VECTOR = 128; // query rows the fp32 vector kernel handles per pass (and its tile size)
constexpr int LONG_N = 1 << 18; // from this sequence length on the MFMA kernel uses 8-wavefront work-groups (256-row tiles)
constexpr int LONG_N_TWO_PASS = 1 << 17; // ... and from this length on where the attention launch runs as two passes
constexpr int KT = 64;         // keys per attention tile; class segments of the permuted keys are padded to this
constexpr int MAX_CLASSES = 256;
constexpr int MAX_HQ = 256;
constexpr int KN2_SLOTS = 64;  // partial maxima of the squared key norms per (batch, KV head), one per lane of a wavefront
constexpr int KPOS_PAD = 0x7fffffff;  // position stored in padded key slots: never <= a query position

// Element types as the kernels see them: float, uint16_t for a bfloat16 bit pattern, f16_bits for an IEEE half.
struct f16_bits { uint16_t v; };
// Direct global -> LDS load of one wavefront: lane l fetches the 16 bytes at (sbase + voff) into LDS byte address
// lds_addr + 16*l (global_load_lds_dwordx4; sbase and lds_addr wave-uniform, voff per lane).  Counted by vmcnt
// like any vector memory load: `s_waitcnt vmcnt(0)` before the data is read from LDS.
__device__ inline void lds_dma16(const void* sbase, unsigned voff, unsigned lds_addr)
{
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 :: "v"(voff), "s"(sbase), "s"(lds_addr) : "memory");
}
// LDS byte address of a __shared__ object (the low half of its generic address)
__device__ inline unsigned lds_addr_of(const void* p) { return (unsigned)(uintptr_t)p; }

__device__ inline float f16_bits_to_f32(uint16_t b)
{
    _Float16 h;
    __builtin_memcpy(&h, &b, 2);
    return (float)h;
}
__device__ inline uint16_t f32_to_f16_bits(float f)
{
    const _Float16 h = (_Float16)f;                     // round to nearest even
    uint16_t b;
    __builtin_memcpy(&b, &h, 2);
    return b;
}

struct HeadMap {               // query head -> KV head, passed by value to kernels
    uint8_t kv[MAX_HQ];
};

// Everything the kernels need to know about shapes and where things live in the
// workspace (byte offsets from its base, all multiples of 256).
struct Layout {
    int B, Hq, Hkv, n, d;
    int K, topk, window;       // window clamped to n
    int causal;                // 1: keys j <= i, local = i-w < j <= i; 0: every j, local = |i-j| < w
    int dtype;                 // 0 fp32, 1 bf16, 2 fp16
    int elem;                  // bytes per element
    int dp;                    // row length of the class-ordered K / V^T copies: d rounded up to 64, 128 or 256
    int BQ;                    // query rows per attention tile (128; 256 for 16-bit types at n >= LONG_N, d <= 128)
    int NC;                    // number of membership classes (1 in dense mode)
    int dense;                 // every causal pair allowed: one class, no masks beyond causal
    int soft;                  // Sec. 2 Eq. 2: every causal pair, the logit of a pair outside the window scaled by
    float gate_slope;          // sigmoid(lambda * g_i . g_j); gate_slope = -lambda * log2(e).  One class, position order.
    int coarse;                // C(K,topk) exceeds MAX_CLASSES: classes are sets of S super-groups (group g folds
    int S;                     // onto g % S), a superset test; the kernels then test the real masks per pair
    int pair_set;              // which pairs a launch attends: 0 the whole mask, 1 only pairs that share a group
                               // (set A of App. D), 2 only window pairs that share none (set B), 3 pairs that share
                               // a group and lie outside the window (second pass of a two-pass launch)
    int two_pass;              // the whole-mask attention launch of this problem runs as two passes: every pair inside
                               // the window over position-ordered rows and keys (the embedded local layout), then the
                               // pairs outside the window that share a group over class-ordered ones, merged per row
    int class_major;           // job list of the attention launch by class (long sequences) instead of by slot
    int local_only;            // this IS the embedded local layout: one class in position order, window pairs only
    int merge_prev;            // launch flag of the second pass: out / lse / row_pairs hold the first pass's partial
                               // result of every row; merge instead of overwriting (App. D's log-sum-exp merge)
    int nblk;                  // ceil(n / SB)
    int NQP;                   // padded per-head length of the class-ordered query index
    int NKP;                   // padded per-head length of the class-ordered key arrays (multiple of KT)
    int NT;                    // upper bound of query tiles per head
    float scale;
    float softcap;

    long long qs[3], ks[3], os[3];     // strides of q, of k and v, of out in elements (batch, head, position)

    size_t off_mq, off_mk;
    size_t off_qgc, off_kgc;           // group counts
    size_t off_qgl, off_kgl;           // group lists
    size_t off_qgo, off_kgo;           // group list offsets [.,K+1]
    size_t off_qcls, off_kcls;         // class id per position, uint8
    size_t off_qbc, off_kbc;           // per sort block class histogram -> exclusive prefix [.,nblk,NC]
    size_t off_qbg, off_kbg;           // per sort block group histogram -> exclusive prefix [.,nblk,K]
    size_t off_qcc, off_kcc;           // class counts [.,NC]
    size_t off_qco, off_kco;           // padded class offsets [.,NC+1]
    size_t off_clsmask;                // group bit mask of each class [NC]
    size_t off_cent64;                 // centroids as fp64 [Hkv][d rounded up to whole 128-byte row chunks][KMAX],
                                       // KMAX = K rounded up to 4/8/16/32
    size_t off_qperm;                  // [B,Hq,NQP] positions in class order, -1 in pads (the scatter kernel writes both)
    size_t off_kpos;                   // [B,Hkv,NKP] positions in class order, KPOS_PAD in pads
    size_t off_kmsk;                   // [B,Hkv,NKP] membership masks in class order, 0 in pads (coarse classes only)
    size_t off_jobs;                   // [B,Hq,NT] (class << 24 | tile) heaviest first, -1 unused
    size_t off_gk;                     // [B,NKP,2,32] bf16: the soft assignment of every key position as bf16 high and
                                       // low parts, groups padded to 32, chunks swizzled per key (soft gate, 16-bit types)
    size_t off_kn2;                    // [B,Hkv,KN2_SLOTS] bit patterns of partial maxima of the squared key norms of the
                                       // head (16-bit types; cleared by assign_init, raised by the scatter kernel's key
                                       // copy, the attention kernel takes the largest)
    size_t off_local;                  // the embedded local layout's own workspace (two_pass)
    size_t off_lse1;                   // [B,Hq,n] fp32: log-sum-exp of the first pass when the caller passes no lse (two_pass)
    size_t off_nrflag;                 // [B,Hq,NT] per work-group of the attention launch: 1 = the no-reference
                                       // instantiation did the tile, 0 = left to the other one (16-bit types)
    size_t off_kc;                     // [B,Hkv,NKP,dp] keys in class order (16-bit types)
    size_t off_vt;                     // [B,Hkv,NKP/KT,dp,KT] values, transposed per key tile (16-bit types)
    size_t total;
};

// colex rank of the k-subset `m` among all k-subsets (device + host)
__host__ __device__ inline uint32_t binom_u32(int a, int b)
{
    if (b < 0 || b > a) return 0;
    if (b > a - b) b = a - b;
    uint64_t r = 1;
    for (int i = 1; i <= b; ++i) r = r * (uint64_t)(a - b + i) / (uint64_t)i;
    return (uint32_t)r;
}

// Coarse classes: the S-bit set of super-groups a membership mask folds onto
__host__ __device__ inline uint32_t fold_groups(uint32_t mask, int S)
{
    uint32_t r = 0;
    while (mask) {
        const int g = __builtin_ctz(mask);
        r |= 1u << (g % S);
        mask &= mask - 1;
    }
    return r;
}

// Class id of a membership mask.  Exact classes: the colex rank of the topk-subset of the K groups.
// Coarse classes: the folded set has 1..topk members; sets are ordered by size, then colex.
__host__ __device__ inline int class_of_mask(uint32_t mask, int dense, int coarse, int S)
{
    if (dense) return 0;
    uint32_t m = coarse ? fold_groups(mask, S) : mask;
    int j = 0, cls = 0;
    while (m) {
        const int g = __builtin_ctz(m);
        ++j;
        cls += (int)binom_u32(g, j);
        m &= m - 1;
    }
    if (coarse)
        for (int t = 1; t < j; ++t) cls += (int)binom_u32(S, t);
    return cls;
}

// Shapes and workspace offsets of the router (focus_route).
struct RouteLayout {
    int B, n, dm, dg, K, topk;
    int dtype;                 // of the hidden states: 0 fp32, 1 bf16
    int iters;                 // Sinkhorn rounds, 0 = none
    double tau;
    int nproj;                 // work-groups of the projection per sequence = ceil(n / 64)
    int nsink;                 // work-groups of a Sinkhorn pass per sequence (<= 256)
    int sink_tokens;           // tokens per Sinkhorn work-group
    size_t off_w64;            // W_g as fp64 [dm][dg]
    size_t off_c64;            // C as fp64 [K][dg]
    size_t off_S;              // [B][n][K] fp64: scores, then exp((S - max)/tau) in place
    size_t off_maxpart;        // [B][nproj] fp64
    size_t off_smax;           // [B] fp64
    size_t off_colpart;        // [2][B][nsink][KP] fp64 column partial sums, ping-pong between passes
    size_t total;
};

// Shapes and state offsets of the incremental (one token per step) path.
#ifndef FOCUS_DEC_CHUNK
#define FOCUS_DEC_CHUNK 512
#endif
constexpr int DEC_CHUNK = FOCUS_DEC_CHUNK;   // keys of the key sequence a work-group of the decode attention resolves at a time
constexpr int DEC_CHUNK_SHORT = 128;         // ... in launches that would otherwise leave most of the chip idle (128 or 256)
static_assert(DEC_CHUNK == 4 * DEC_CHUNK_SHORT, "the launch picks among DEC_CHUNK_SHORT, twice that, and DEC_CHUNK");
constexpr int DEC_MAX_PARTS = 384;           // partial results per head the merge reads at most
struct DecodeLayout {
    int B, Hq, Hkv, n, d;      // n = capacity of the caches
    int K, topk, window;
    int dtype;
    float scale, softcap;
    int max_chunks;            // chunks of DEC_CHUNK keys the longest key sequence (n entries) has
    int max_parts;             // partial results per head: min(chunks of DEC_CHUNK_SHORT keys, DEC_MAX_PARTS)
    size_t off_mk;             // [B,Hkv,n] uint32 membership of the cached keys
    size_t off_lists;          // [B,Hkv,K,n] int32 positions of every group, ascending
    size_t off_counts;         // [B,Hkv,K] int32 list lengths
    size_t off_wp;             // [B,Hkv,K] int32 list entries below the current step's window
    size_t off_mq;             // [B,Hq] uint32 membership of the current queries
    size_t off_part;           // [B,Hq,max_parts,d+4] fp32 partial (o, max, sum, count) per work-group
    size_t total;
};

// token_masks / token_mask non-NULL: memberships given per token (centroids unused) instead of scored per head
hipError_t launch_decode_prefill(const DecodeLayout& L, int n_ctx, const void* kc, const float* cents,
                                 const uint32_t* token_masks, char* st, hipStream_t s);
hipError_t launch_decode_step(const DecodeLayout& L, const HeadMap& hm, int pos, const int* pos_dev, const void* q_new, const void* k_new,
                              const void* v_new, const float* cents, const uint32_t* token_mask, void* kc, void* vc, char* st,
                              void* out, float* lse, int32_t* row_pairs, hipStream_t s);
hipError_t launch_route(const RouteLayout& R, const void* hidden, const float* wg, const float* cent, char* ws,
                        uint32_t* masks, double* soft, hipStream_t st);
// The router's scratch for callers that may not allocate: a buffer of ROUTE_STATIC_SCRATCH_BYTES that lives in
// the library's device image; *ptr is its address on the CURRENT device (looked up once per device).
constexpr size_t ROUTE_STATIC_SCRATCH_BYTES = (size_t)16 << 20;
hipError_t route_static_scratch(char** ptr);
hipError_t launch_assign_tokens(const Layout& L, const uint32_t* token_masks, const void* k, char* ws,
                                int32_t* invalid_count, hipStream_t st);
hipError_t launch_assign(const Layout& L, const HeadMap& hm, const void* q, const void* k,
                         const float* centroids, char* ws, hipStream_t st);
hipError_t launch_attn_simple(const Layout& L, const HeadMap& hm, const void* q, const void* k,
                              const void* v, const float* g, char* ws, void* out, float* lse, int32_t* row_pairs,
                              hipStream_t st);
hipError_t launch_soft_gather_g(const Layout& L, const float* g, char* ws, hipStream_t st);
hipError_t launch_attn_merge(size_t rows, int d, int dtype, const void* oa, const float* la, const void* ob,
                             const float* lb, void* out, float* lse, hipStream_t st);
hipError_t launch_attn_mfma(const Layout& L, const HeadMap& hm, const void* q, const void* k,
                            const void* v, const float* g, char* ws, void* out, float* lse, int32_t* row_pairs,
                            hipStream_t st);

}  // namespace focus
