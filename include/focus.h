/*
 * focus.h -- C ABI of libfocus.so: the group-gated sparse attention forward of
 * "Composing Sparse Attention via Learned Grouping" (Focus) on one MI355X.
 *
 * Two calls make the hot path:
 *   focus_assign    scores every query and key vector against K centroids per
 *                   head (Sec. 2, Eq. 1, in the per-head dot-product form),
 *                   keeps each token's top-k groups (Sec. 2 "Efficiency at
 *                   inference", Sec. 3.6), and buckets tokens by group in
 *                   ascending position (the stable sort of App. D);
 *   focus_attn_fwd  exact-softmax attention over the pairs that App. D Eq. 3
 *                   allows, generalised to top-k sets: pair (i,j) is attended
 *                   iff j <= i and (i - j < window or the two membership sets
 *                   intersect); each allowed pair enters one softmax once.
 *
 * Conventions
 *   - extern "C", no exceptions, no torch types.  Every call returns a
 *     focus_status; focus_last_error() gives the message of the last failure on
 *     the calling thread.
 *   - q, k, v, out, centroids, workspace, lse, row_pairs are DEVICE pointers of
 *     the current HIP device; `p` and p->head_map are HOST pointers.
 *   - q, out: [B,Hq,n,d]; k, v: [B,Hkv,n,d]; d innermost and contiguous, the other
 *     three indices strided (focus_params), contiguous by default; 16-byte
 *     aligned.  centroids: [Hkv,K,d] fp32 (used as given, never renormalised).
 *   - The caller owns all buffers.  The library allocates no device memory and
 *     keeps no state between calls.  The workspace is caller-allocated,
 *     256-byte aligned, at least focus_workspace_size() bytes, and carries the
 *     result of focus_assign to focus_attn_fwd (same params, same k).  Both
 *     calls WRITE it: focus_assign fills the membership, the lists, the schedule
 *     and the class-ordered copy of the keys; focus_attn_fwd (and its variants)
 *     adds the class-ordered, transposed copy of the values before its attention
 *     launch, so v may change between two attention calls on one workspace, while
 *     k may not.  Two attention calls that share a workspace must not overlap.
 *   - focus_assign and focus_attn_fwd only enqueue work on `stream`
 *     (a hipStream_t passed as void*, NULL = default stream) and return; the
 *     caller synchronises.  Inputs are never modified; out must not alias them.
 *   - Argument errors are detected on the host before anything is launched.
 *     Non-finite inputs give undefined results.
 */
#ifndef FOCUS_H
#define FOCUS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    FOCUS_OK = 0,
    FOCUS_EINVAL = -1,        /* bad argument (NULL pointer, range, alignment) */
    FOCUS_EUNSUPPORTED = -2,  /* valid request this build has no kernel for    */
    FOCUS_EWORKSPACE = -3,    /* workspace too small or misaligned             */
    FOCUS_EHIP = -4           /* a HIP call failed (launch error text kept)    */
} focus_status;

typedef enum { FOCUS_F32 = 0, FOCUS_BF16 = 1, FOCUS_F16 = 2 } focus_dtype;   /* F16 = IEEE binary16 */

typedef struct {
    int32_t B, Hq, Hkv, n, d;  /* d in {64,80,96,128,256}; Hq % Hkv == 0 unless
                                  head_map                                       */
    int32_t K, topk;           /* 1 <= topk <= K <= 32 groups per KV head        */
    int32_t window;            /* w >= 1: the local keys of query i are i-w < j <= i
                                  (w keys including the query itself) when causal,
                                  |i-j| < w when not; w >= n means plain attention */
    int32_t causal;            /* 1: keys j <= i only; 0: keys on both sides (the
                                  incremental path takes 1 only)                 */
    int32_t dtype;             /* focus_dtype of q, k, v, out                    */
    float scale;               /* logit scale, 0 selects 1/sqrt(d) (Sec. 2)      */
    float softcap;             /* 0 = off, else logit = softcap*tanh(scale*q.k/softcap),
                                  applied before masking                         */
    const int32_t *head_map;   /* HOST [Hq] query head -> KV head (keys, values,
                                  key membership and centroids); NULL selects
                                  h / (Hq / Hkv)                                 */
    /* Strides of q, of k and v (both the same) and of out, in ELEMENTS, for the batch, head and
     * position index; the d components of a row are contiguous.  All three 0 selects the contiguous
     * [B,H,n,d]; a [B,n,H,d] tensor is {n*H*d, d, H*d}.  Every stride must be a multiple of 16 bytes.
     * The prefill path (focus_assign, focus_assign_tokens, focus_attn_fwd, focus_attn_fwd_set,
     * focus_attn_soft_fwd) takes strides; the two-call convenience and the incremental path take
     * contiguous tensors only (FOCUS_EUNSUPPORTED otherwise). */
    int64_t q_strides[3];
    int64_t kv_strides[3];
    int64_t o_strides[3];
} focus_params;

/* Bytes of workspace the two calls need for these params.  Pure host code. */
focus_status focus_workspace_size(const focus_params *p, size_t *bytes);

/* Sec. 2 Eq. 1 + top-k + bucketing.  Fills the workspace: membership bit masks
 * (bit g = token belongs to group g; ties in the top-k go to the smaller group
 * index; scores are the fp64 dot products accumulated in index order), per-group
 * counts and position-ascending index lists, and the internal schedule that
 * focus_attn_fwd consumes. */
focus_status focus_assign(const focus_params *p, const void *q, const void *k,
                          const float *centroids, void *workspace,
                          size_t workspace_bytes, void *stream);

/* App. D Eq. 3 with top-k sets, exact softmax (Sec. 1), after focus_assign on
 * the same workspace.  For 16-bit causal problems of n >= 16384 whose window spans
 * would be mostly masked in class-ordered tiles, the launch runs as two passes
 * (the pairs inside the window over position-ordered tiles, then the pairs outside
 * it that share a group over class-ordered tiles) and merges the two partial
 * softmaxes of every row through their log-sum-exp (App. D's merge): the same exact
 * softmax, each allowed pair once; focus_workspace_size and focus_assign account
 * for the second layout.  The environment variable FOCUS_TWO_PASS=0/1, read when a
 * call derives its layout, overrides that choice (tests and measurements; it must
 * not change between focus_workspace_size, focus_assign and focus_attn_fwd).  out [B,Hq,n,d] in p->dtype.  lse (nullable) [B,Hq,n]
 * fp32: natural log of the sum of exp of the final logits of the row.
 * row_pairs (nullable) [B,Hq,n] int32: number of pairs the row attended.  The
 * workspace is written (staging of V). */
focus_status focus_attn_fwd(const focus_params *p, const void *q, const void *k,
                            const void *v, void *workspace, size_t workspace_bytes,
                            void *out, float *lse, int32_t *row_pairs, void *stream);

/* focus_attn_fwd (same contract, same checks) forced through the fp32 vector-ALU kernel in every dtype:
 * no matrix cores, slow.  It exists so that tests can cross-check the matrix-core kernel on the device at
 * sizes a CPU reference cannot cover in full; it is not part of the hot path (App. D Eq. 3, as above). */
focus_status focus_attn_fwd_vector(const focus_params *p, const void *q, const void *k,
                                   const void *v, void *workspace, size_t workspace_bytes,
                                   void *out, float *lse, int32_t *row_pairs, void *stream);

/* ---- the soft-gated attention of training (Sec. 2 Eq. 2) ----
 *
 * Every causal pair is computed: logit_ij = scale * q_i.k_j * gate_ij with gate_ij = 1 inside the
 * window (i-w < j <= i) and sigmoid(lambda * g_i.g_j) outside, exact softmax over j <= i, times V.
 * The equation is taken as printed: a gate of sigmoid(0) = 1/2 halves a logit, it removes no pair.
 * g [B,n,K] fp32 DEVICE: the soft assignment of every token of the layer (the same for all heads;
 * focus_route's `soft` output rounded to fp32, or any other); lambda finite.  p->K is the width of g,
 * p->topk is not used (give 1), p->causal must be 1 and p->softcap 0 (else FOCUS_EUNSUPPORTED).
 * One call does everything (no focus_assign): the workspace of focus_soft_workspace_size(p) bytes is
 * scratch (position-ordered copies of K, V and g).  out [B,Hq,n,d] in p->dtype, lse (nullable)
 * [B,Hq,n] fp32.  Forward only.  d = 256 runs on the vector ALUs in every dtype (slow). */
focus_status focus_soft_workspace_size(const focus_params *p, size_t *bytes);
focus_status focus_attn_soft_fwd(const focus_params *p, float lambda, const float *g,
                                 const void *q, const void *k, const void *v, void *workspace,
                                 size_t workspace_bytes, void *out, float *lse, void *stream);
/* The same (Sec. 2 Eq. 2) forced through the vector-ALU kernel: the tests' on-device cross-check. */
focus_status focus_attn_soft_fwd_vector(const focus_params *p, float lambda, const float *g,
                                        const void *q, const void *k, const void *v, void *workspace,
                                        size_t workspace_bytes, void *out, float *lse, void *stream);

/* ---- the per-layer router in front of the attention (Sec. 2 Eq. 1 and the Sinkhorn recipe) ----
 *
 * The paper routes once per layer: a token's hidden state h_i is projected by W_g (d_model x d_g),
 * scored against K centroids of width d_g, optionally Sinkhorn-normalised over the sequence, and its
 * topk best groups are its membership for every head, as a query and as a key. */
typedef struct {
    int32_t B, n;              /* hidden is [B,n,d_model]                              */
    int32_t d_model;           /* multiple of 8                                        */
    int32_t d_g;               /* router width: 4, 8, 16, 32 or 64                     */
    int32_t K, topk;           /* 1 <= topk <= K <= 32                                 */
    int32_t dtype;             /* focus_dtype of hidden                                */
    int32_t sinkhorn_iters;    /* N >= 0; 0 = no normalisation (scores / tau)          */
    double tau;                /* temperature > 0                                      */
} focus_route_params;

/* Bytes of workspace focus_route needs.  Pure host code. */
focus_status focus_route_workspace_size(const focus_route_params *rp, size_t *bytes);

/* z_i = W_g^T h_i, S[i,g] = z_i . C[g] (Sec. 2 Eq. 1), all in fp64: the (exact) products of the
 * projection are added one by one over the hidden components in index order, S over the d_g
 * components in index order.
 * sinkhorn_iters = 0: g_i = S[i,:] / tau.  Otherwise Q = exp((S - max S of the sequence) / tau),
 * then N rounds per batch element of {every column divided by its sum over the n tokens, every
 * row divided by its sum over the K groups} (evaluated as diagonal scalings of Q), g_i = Q[i,:].
 * token_masks [B,n] uint32 receives the topk largest entries of g_i as bits (ties to the smaller
 * group index); soft (nullable) [B,n,K] fp64 receives g itself.
 * hidden, w_g [d_model,d_g] fp32, centroids [K,d_g] fp32, route_workspace (256-byte aligned),
 * token_masks and soft are DEVICE pointers; rp is a HOST pointer.  Only enqueues on `stream`.
 * Scores so far apart that a whole row or column of Q underflows give NaN rows, as the
 * recipe itself does. */
focus_status focus_route(const focus_route_params *rp, const void *hidden, const float *w_g,
                         const float *centroids, void *route_workspace, size_t workspace_bytes,
                         uint32_t *token_masks, double *soft, void *stream);

/* focus_route for callers that cannot allocate device memory or hand over a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, checks, kernels and
 * results as focus_route, but the scratch is a buffer inside the library's own device image (16 MiB per GPU,
 * held until the process ends) instead of route_workspace; the call allocates nothing.  A problem whose
 * focus_route_workspace_size() exceeds 16 MiB (about B*n*K*8 + d_model*d_g*8 bytes: e.g. n = 131072 with
 * K = 8 still fits, n = 262144 with K = 8 does not) is refused with FOCUS_EWORKSPACE before anything is
 * launched.  All calls on one GPU share that one buffer: two calls that overlap in time on the same GPU
 * (different streams or threads) race; calls on one stream are safe back to back.  Nothing in the buffer is
 * read before the same call has written it, so leftovers of an earlier call do no harm. */
focus_status focus_route_noalloc(const focus_route_params *rp, const void *hidden, const float *w_g,
                                 const float *centroids, uint32_t *token_masks, double *soft,
                                 void *stream);

/* focus_assign for memberships given per token (the router's output): token_masks [B,n]
 * uint32 DEVICE, each a topk-subset of the K groups, shared by all query and KV heads of
 * the token.  Fills the workspace exactly as focus_assign does (masks, counts, lists,
 * schedule), so focus_attn_fwd follows unchanged.  A mask with another popcount or with
 * bits at or above K is replaced by the first topk groups; invalid_count (nullable, DEVICE
 * int32) receives how many were replaced. */
focus_status focus_assign_tokens(const focus_params *p, const uint32_t *token_masks, const void *k,
                                 void *workspace, size_t workspace_bytes, int32_t *invalid_count,
                                 void *stream);

/* ---- the paper's two-call evaluation (App. D), as a measured comparator of the fused kernel ----
 *
 * App. D splits the mask into two disjoint sets, A = causal pairs of the same group and
 * B = causal pairs inside the window of different groups, evaluates each with its own softmax
 * and merges the two results through their log-sum-exp values.  With top-k sets: A = pairs whose
 * membership sets intersect, B = window pairs whose sets do not.  These calls run after
 * focus_assign (or focus_assign_tokens) on the same workspace, like focus_attn_fwd. */
typedef enum { FOCUS_PAIRS_ALL = 0, FOCUS_PAIRS_SHARED = 1, FOCUS_PAIRS_CROSS_LOCAL = 2 } focus_pair_set;

/* focus_attn_fwd restricted to one pair set.  A row with no pair in the set gets out = 0,
 * lse = -inf, row_pairs = 0.  FOCUS_EUNSUPPORTED for a restricted set when window >= n. */
focus_status focus_attn_fwd_set(const focus_params *p, int32_t pair_set, const void *q, const void *k,
                                const void *v, void *workspace, size_t workspace_bytes, void *out,
                                float *lse, int32_t *row_pairs, void *stream);

/* App. D "Merge": out = (e^{lse_a} out_a + e^{lse_b} out_b) / (e^{lse_a} + e^{lse_b}) per row and
 * lse (nullable) = log(e^{lse_a} + e^{lse_b}); rows of d components (a multiple of 8) in dtype,
 * lse fp32; all DEVICE pointers, 16-byte aligned; out may alias out_a or out_b. */
focus_status focus_attn_merge(int64_t rows, int32_t d, int32_t dtype, const void *out_a,
                              const float *lse_a, const void *out_b, const float *lse_b, void *out,
                              float *lse, void *stream);

/* Set A, set B, merge: three launches on `stream`.  part_out: DEVICE scratch of 2 x [B,Hq,n,d]
 * elements of p->dtype, part_lse: DEVICE scratch of 2 x [B,Hq,n] fp32, both caller-owned. */
focus_status focus_attn_fwd_two_call(const focus_params *p, const void *q, const void *k,
                                     const void *v, void *workspace, size_t workspace_bytes,
                                     void *out, float *lse, void *part_out, float *part_lse,
                                     void *stream);

/* ---- incremental inference: one new token per sequence against a key/value cache ----
 *
 * The paper evaluates generation (Sec. 3.3) but does not describe a decode kernel; this is the same
 * mask row (App. D Eq. 3 with top-k sets) for the newest token i: keys j <= i with i - j < window or
 * with a membership set that intersects the query's.  p->n is the CAPACITY of the caches
 * k_cache, v_cache [B,Hkv,n,d] (DEVICE, p->dtype, 16-byte aligned).  `state` is caller-allocated
 * DEVICE memory of focus_decode_state_size() bytes, 256-byte aligned: the membership mask of every
 * cached key, one ascending position list per (batch, KV head, group), and scratch for the step.
 * K up to 32 with any topk (no limit on the number of membership classes here). */
focus_status focus_decode_state_size(const focus_params *p, size_t *bytes);

/* Builds the state for the first n_ctx (0 <= n_ctx <= n) rows already in k_cache: scores every
 * cached key against the centroids [Hkv,K,d] (fp64, index order, ties to the smaller group) and
 * fills masks and lists.  Enqueues on `stream`. */
focus_status focus_decode_prefill(const focus_params *p, int32_t n_ctx, const void *k_cache,
                                  const float *centroids, void *state, size_t state_bytes,
                                  void *stream);

/* One step at position pos (the positions 0 .. pos-1 are in the caches and in the state; steps must
 * come in order and calls on one state must not overlap): routes k_new [B,Hkv,d] and q_new
 * [B,Hq,d], stores k_new and v_new [B,Hkv,d] at row pos of the caches, appends pos to the lists of
 * the key's groups, then attends.  out [B,Hq,d] in p->dtype; lse (nullable) [B,Hq] fp32;
 * row_pairs (nullable) [B,Hq] int32 = keys attended.  Three launches on `stream`. */
focus_status focus_decode_step(const focus_params *p, int32_t pos, const void *q_new,
                               const void *k_new, const void *v_new, const float *centroids,
                               void *k_cache, void *v_cache, void *state, size_t state_bytes,
                               void *out, float *lse, int32_t *row_pairs, void *stream);

/* The paper's per-layer routing in the incremental path: memberships are given per token (focus_route's
 * masks; at inference without the Sinkhorn rounds, which need the whole sequence) instead of scored per head.
 * focus_decode_prefill_tokens builds the state from token_masks [B, n_ctx] uint32 DEVICE (every KV head of a
 * token takes the token's mask; k_cache is not read).  focus_decode_step_tokens takes the new token's mask,
 * token_mask [B] uint32 DEVICE, for all its query heads and as its key.  A mask that is not a topk-subset of
 * the K groups is replaced by the first topk groups.  Everything else as in focus_decode_step. */
focus_status focus_decode_prefill_tokens(const focus_params *p, int32_t n_ctx, const uint32_t *token_masks,
                                         void *state, size_t state_bytes, void *stream);
focus_status focus_decode_step_tokens(const focus_params *p, int32_t pos, const uint32_t *token_mask,
                                      const void *q_new, const void *k_new, const void *v_new,
                                      void *k_cache, void *v_cache, void *state, size_t state_bytes,
                                      void *out, float *lse, int32_t *row_pairs, void *stream);

/* The same step with the positions read from DEVICE memory by the kernels when they run:
 * pos_dev [B] int32, one position per sequence.  A HIP graph captured once around this call serves every
 * step of a generation loop (the caller writes the new tokens' q, k, v into the captured buffers and
 * advances pos_dev on the device between replays), and the sequences of a batch may stand at different
 * positions.  A sequence whose position is outside [0, n) is skipped: its caches, state and outputs stay
 * untouched (a finished or not yet started sequence of a continuous batch; the host cannot check device
 * values).  The launch shapes are those of the last position the caches can hold; work-groups past a
 * sequence's real length exit at once. */
focus_status focus_decode_step_at(const focus_params *p, const int32_t *pos_dev, const void *q_new,
                                  const void *k_new, const void *v_new, const float *centroids,
                                  void *k_cache, void *v_cache, void *state, size_t state_bytes,
                                  void *out, float *lse, int32_t *row_pairs, void *stream);

/* Device pointers INTO the decode state for parity checks (any may be NULL): mk [B,Hkv,n] uint32
 * masks of the cached keys, lists [B,Hkv,K,n] int32 (the first counts[b,h,g] entries of a list are
 * its positions, ascending), counts [B,Hkv,K] int32, mq [B,Hq] uint32 masks of the last step's queries. */
focus_status focus_decode_state_views(const focus_params *p, void *state, const uint32_t **mk,
                                      const int32_t **lists, const int32_t **counts,
                                      const uint32_t **mq);

/* Device pointers INTO the workspace for parity checks; valid until the
 * workspace is overwritten.  Any output pointer may be NULL.
 *   mq [B,Hq,n], mk [B,Hkv,n]                   uint32 membership masks
 *   q_group_counts [B,Hq,K], k_group_counts [B,Hkv,K]
 *   q_group_lists [B,Hq,topk*n], k_group_lists [B,Hkv,topk*n]: per (b,h) the
 *     lists of group 0,1,.. back to back, each position-ascending. */
focus_status focus_workspace_views(const focus_params *p, void *workspace,
                                   const uint32_t **mq, const uint32_t **mk,
                                   const int32_t **q_group_counts,
                                   const int32_t **k_group_counts,
                                   const int32_t **q_group_lists,
                                   const int32_t **k_group_lists);

/* Message of the last failure on this thread (static storage, never NULL). */
const char *focus_last_error(void);

/* major*10000 + minor*100 + patch */
int focus_version(void);

/* Identifier of the sources this library was compiled from (a hash the build computes over them;
 * "unknown" when built by hand).  The Python binding refuses to run a library older than its sources. */
const char *focus_build_id(void);

#ifdef __cplusplus
}
#endif
#endif /* FOCUS_H */
