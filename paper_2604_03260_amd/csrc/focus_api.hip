// Host side of libfocus.so: argument checks, workspace layout, dispatch.
// Everything that computes runs in the HIP kernels of the other translation units.
// the library is compiled with hidden visibility: only what the public header declares is exported
#pragma GCC visibility push(default)
#include "../../include/focus.h"
#pragma GCC visibility pop
#include "focus_internal.h"

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>

namespace {

thread_local char g_err[512] = "no error";

focus_status fail(focus_status st, const char* fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return st;
}

size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

// true when q, k/v and out are the contiguous [B,H,n,d] (strides all zero, or spelled out)
bool contiguous_tensors(const focus_params* p)
{
    const int64_t* src[3] = {p->q_strides, p->kv_strides, p->o_strides};
    const int heads[3] = {p->Hq, p->Hkv, p->Hq};
    for (int t = 0; t < 3; ++t) {
        if (src[t][0] == 0 && src[t][1] == 0 && src[t][2] == 0) continue;
        if (src[t][0] != (int64_t)heads[t] * p->n * p->d || src[t][1] != (int64_t)p->n * p->d || src[t][2] != p->d)
            return false;
    }
    return true;
}

// Validates the params and derives the workspace layout and the head map.
// soft: the layout of the soft-gated attention (one class in position order whatever K, topk and the window are).
// local: the position-ordered second layout that a two-pass problem embeds in its workspace.
focus_status make_layout(const focus_params* p, focus::Layout* L, focus::HeadMap* hm, bool soft = false, bool local = false)
{
    using namespace focus;
    if (!p) return fail(FOCUS_EINVAL, "params is NULL");
    if (p->B < 1 || p->Hq < 1 || p->Hkv < 1 || p->n < 1)
        return fail(FOCUS_EINVAL, "B, Hq, Hkv, n must be >= 1 (got %d %d %d %d)", p->B, p->Hq, p->Hkv, p->n);
    if (p->dtype != FOCUS_F32 && p->dtype != FOCUS_BF16 && p->dtype != FOCUS_F16)
        return fail(FOCUS_EINVAL, "unknown dtype %d", p->dtype);
    if (p->K < 1 || p->K > 32) return fail(FOCUS_EINVAL, "K must be in [1,32] (got %d)", p->K);
    if (p->topk < 1 || p->topk > p->K)
        return fail(FOCUS_EINVAL, "topk must be in [1,K] (got %d, K=%d)", p->topk, p->K);
    if (p->window < 1) return fail(FOCUS_EINVAL, "window must be >= 1 (got %d)", p->window);
    if (p->causal != 0 && p->causal != 1) return fail(FOCUS_EINVAL, "causal must be 0 or 1");
    if (!(p->scale >= 0.0f) || !std::isfinite(p->scale))
        return fail(FOCUS_EINVAL, "scale must be finite and >= 0");
    if (!(p->softcap >= 0.0f) || !std::isfinite(p->softcap))
        return fail(FOCUS_EINVAL, "softcap must be finite and >= 0");
    if (p->d < 1) return fail(FOCUS_EINVAL, "d must be >= 1");
    if (p->head_map) {
        for (int h = 0; h < p->Hq; ++h)
            if (p->head_map[h] < 0 || p->head_map[h] >= p->Hkv)
                return fail(FOCUS_EINVAL, "head_map[%d]=%d is outside [0,Hkv)", h, p->head_map[h]);
    } else if (p->Hq % p->Hkv != 0) {
        return fail(FOCUS_EINVAL, "Hq (%d) is not a multiple of Hkv (%d) and no head_map given", p->Hq, p->Hkv);
    }
    // valid, but no kernel in this build
    if (p->d != 64 && p->d != 80 && p->d != 96 && p->d != 128 && p->d != 256)
        return fail(FOCUS_EUNSUPPORTED, "head dim %d is not built (64, 80, 96, 128 or 256)", p->d);
    if (p->Hq > MAX_HQ || p->Hkv > MAX_HQ)
        return fail(FOCUS_EUNSUPPORTED, "more than %d heads is not built", MAX_HQ);
    if (p->n > (1 << 24)) return fail(FOCUS_EUNSUPPORTED, "n above 2^24 is not built");
    if ((int64_t)p->B * p->Hq > 65535 || (int64_t)p->B * p->Hkv > 65535)
        return fail(FOCUS_EUNSUPPORTED, "B*H above 65535 is not built");

    memset(L, 0, sizeof(*L));
    L->B = p->B; L->Hq = p->Hq; L->Hkv = p->Hkv; L->n = p->n; L->d = p->d;
    L->K = p->K; L->topk = p->topk; L->window = std::min(p->window, p->n);
    L->causal = p->causal;
    L->dtype = p->dtype;
    L->elem = (p->dtype == FOCUS_F32) ? 4 : 2;
    L->scale = (p->scale > 0.0f) ? p->scale : (float)(1.0 / std::sqrt((double)p->d));
    L->softcap = p->softcap;
    L->soft = soft ? 1 : 0;
    L->local_only = local ? 1 : 0;
    L->dense = (soft || local || p->window >= p->n || 2 * p->topk > p->K) ? 1 : 0;
    if (L->dense) {
        L->NC = 1;
    } else {
        uint64_t c = 1;
        int kk = p->topk;
        for (int i = 1; i <= kk; ++i) {
            c = c * (uint64_t)(p->K - kk + i) / (uint64_t)i;
            if (c > (uint64_t)MAX_CLASSES) break;
        }
        L->NC = (int)c;
        L->S = p->K;
        if (c > (uint64_t)MAX_CLASSES) {
            // too many exact classes: fold the groups onto the largest number S of super-groups whose sets of
            // 1..topk members still fit the class tables
            L->coarse = 1;
            int best = 1, best_nc = 1;
            for (int S = 1; S <= p->K; ++S) {
                uint64_t tot = 0;
                for (int j = 1; j <= std::min(kk, S); ++j) tot += focus::binom_u32(S, j);
                if (tot <= (uint64_t)MAX_CLASSES) { best = S; best_nc = (int)tot; }
            }
            L->S = best;
            L->NC = best_nc;
        }
    }
    // strides: all zero = contiguous [B,H,n,d]; else positive, rows 16-byte aligned, inside int64
    {
        const int64_t* src[3] = {p->q_strides, p->kv_strides, p->o_strides};
        long long* dst[3] = {L->qs, L->ks, L->os};
        const int heads[3] = {p->Hq, p->Hkv, p->Hq};
        const char* names[3] = {"q_strides", "kv_strides", "o_strides"};
        const long long align = 16 / L->elem;
        for (int t = 0; t < 3; ++t) {
            if (src[t][0] == 0 && src[t][1] == 0 && src[t][2] == 0) {
                dst[t][0] = (long long)heads[t] * p->n * p->d;
                dst[t][1] = (long long)p->n * p->d;
                dst[t][2] = p->d;
                continue;
            }
            for (int e = 0; e < 3; ++e) {
                if (src[t][e] <= 0 || src[t][e] % align != 0 || src[t][e] > ((int64_t)1 << 40))
                    return fail(FOCUS_EINVAL, "%s[%d] = %lld must be positive and a multiple of %lld elements (16 bytes)",
                                names[t], e, (long long)src[t][e], align);
                dst[t][e] = src[t][e];
            }
            if (dst[t][2] < p->d) return fail(FOCUS_EINVAL, "%s[2] is smaller than d: rows overlap", names[t]);
        }
    }
    L->nblk = (p->n + SB - 1) / SB;
    // bf16 at long n: 256-row tiles (8 wavefronts share every K/V tile: half the L2->LDS traffic per FLOP,
    // which is what bounds the kernel once a KV head's K/V no longer sits in L2/MALL)
    L->dp = (p->d <= 64) ? 64 : (p->d <= 128) ? 128 : 256;
    const bool can256 = p->dtype != FOCUS_F32 && p->d <= 128 && !L->coarse && !soft;   // shapes with an 8-wavefront kernel
    L->BQ = (can256 && p->n >= LONG_N) ? 256 : BQ_VECTOR;
    // Two passes (see attn_launch) where the rows of a class tile spread over so many positions that the window
    // spans of the classes without a common group, rectangles of key tiles around a diagonal band, would be mostly
    // masked: estimated share of wasted matrix work = (window pairs among all pairs) x spread / (window + spread)
    // with uniform memberships; from 4 % on, and only where the second set of launches is small change (n >= 16384).
    if (!soft && !local && !L->dense && !L->coarse && p->causal && p->dtype != FOCUS_F32) {
        double none = 1.0;                                   // C(K-k, k) / C(K, k): P(two topk-subsets of K do not meet)
        for (int i = 0; i < p->topk; ++i) none *= (double)(p->K - p->topk - i) / (double)(p->K - i);
        const double w = (double)L->window, spread = (double)L->NC * L->BQ;
        const double local_share = w / (0.5 * p->n * (1.0 - none) + w);
        const char* force = getenv("FOCUS_TWO_PASS");        // "0" / "1": override of the estimate (tests, measurements)
        const bool est = p->n >= 16384 && local_share * spread / (w + spread) >= 0.04;
        L->two_pass = (force && (force[0] == '0' || force[0] == '1')) ? (force[0] == '1') : est;
    }
    // With two passes the spread of a tile's rows no longer costs masked work, so the 256-row tiles (every K/V tile
    // fetched feeds twice the rows) pay from 131072 tokens on already (measured: cfg4a 61.8 -> 60.0 ms, cfg4b 177 -> 174 ms)
    if ((L->two_pass || local) && can256 && p->n >= LONG_N_TWO_PASS) L->BQ = 256;
    // class-major launch order only where the heads' K and V are far beyond the caches (see plan_heads_kernel)
    L->class_major = (L->BQ == 256 && p->n >= LONG_N) ? 1 : 0;
    L->NT = (p->n + L->BQ - 1) / L->BQ + L->NC;
    L->NQP = L->NT * L->BQ;
    L->NKP = ((p->n + KT - 1) / KT + L->NC) * KT;

    for (int h = 0; h < p->Hq; ++h)
        hm->kv[h] = (uint8_t)(p->head_map ? p->head_map[h] : h / (p->Hq / p->Hkv));

    const size_t BHq = (size_t)p->B * p->Hq, BHk = (size_t)p->B * p->Hkv;
    const size_t n = (size_t)p->n;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = align256(off + bytes); return o; };
    L->off_mq = take(BHq * n * 4);
    L->off_mk = take(BHk * n * 4);
    L->off_qgc = take(BHq * L->K * 4);
    L->off_kgc = take(BHk * L->K * 4);
    L->off_qgl = take(BHq * n * L->topk * 4);
    L->off_kgl = take(BHk * n * L->topk * 4);
    L->off_qgo = take(BHq * (L->K + 1) * 4);
    L->off_kgo = take(BHk * (L->K + 1) * 4);
    L->off_qcls = take(BHq * n);
    L->off_kcls = take(BHk * ((size_t)L->nblk * SB));
    L->off_qbc = take(BHq * (L->nblk + 1) * L->NC * 4);
    L->off_kbc = take(BHk * (L->nblk + 1) * L->NC * 4);
    L->off_qbg = take(BHq * (L->nblk + 1) * L->K * 4);
    L->off_kbg = take(BHk * (L->nblk + 1) * L->K * 4);
    L->off_qcc = take(BHq * L->NC * 4);
    L->off_kcc = take(BHk * L->NC * 4);
    L->off_qco = take(BHq * (L->NC + 1) * 4);
    L->off_kco = take(BHk * (L->NC + 1) * 4);
    L->off_clsmask = take((size_t)L->NC * 4);
    L->off_cent64 = take((size_t)p->Hkv * (((size_t)p->d * L->elem + 127) / 128 * (128 / L->elem)) * 32 * 8);
    L->off_qperm = take(BHq * L->NQP * 4);
    L->off_kpos = take(BHk * L->NKP * 4);
    L->off_kmsk = L->coarse ? take(BHk * L->NKP * 4) : off;
    L->off_jobs = take(BHq * L->NT * 4);
    L->off_gk = (soft && p->dtype != FOCUS_F32) ? take((size_t)p->B * L->NKP * 128) : off;
    if (L->two_pass) {
        focus::Layout L2;
        focus::HeadMap hm2;
        focus_status st2 = make_layout(p, &L2, &hm2, false, true);
        if (st2 != FOCUS_OK) return st2;
        L->off_local = take(L2.total);
        L->off_lse1 = take(BHq * n * 4);
    }
    L->off_kn2 = take(BHk * focus::KN2_SLOTS * 4);
    L->off_nrflag = take(BHq * L->NT * 4);
    if (p->dtype != FOCUS_F32) {
        L->off_kc = take(BHk * L->NKP * (size_t)L->dp * 2);
        L->off_vt = take(BHk * L->NKP * (size_t)L->dp * 2);
    } else {
        L->off_kc = L->off_vt = off;
    }
    L->total = off;
    return FOCUS_OK;
}

focus_status check_ws(const focus::Layout& L, const void* ws, size_t bytes)
{
    if (!ws) return fail(FOCUS_EINVAL, "workspace is NULL");
    if (((uintptr_t)ws & 255) != 0) return fail(FOCUS_EWORKSPACE, "workspace is not 256-byte aligned");
    if (bytes < L.total)
        return fail(FOCUS_EWORKSPACE, "workspace has %zu bytes, %zu needed", bytes, L.total);
    return FOCUS_OK;
}

bool misaligned16(const void* p) { return ((uintptr_t)p & 15) != 0; }

// Validates the router params and derives its workspace layout.
focus_status make_route_layout(const focus_route_params* rp, focus::RouteLayout* R)
{
    if (!rp) return fail(FOCUS_EINVAL, "route params is NULL");
    if (rp->B < 1 || rp->n < 1) return fail(FOCUS_EINVAL, "B and n must be >= 1 (got %d %d)", rp->B, rp->n);
    if (rp->d_model < 1) return fail(FOCUS_EINVAL, "d_model must be >= 1");
    if (rp->d_g < 1) return fail(FOCUS_EINVAL, "d_g must be >= 1");
    if (rp->K < 1 || rp->K > 32) return fail(FOCUS_EINVAL, "K must be in [1,32] (got %d)", rp->K);
    if (rp->topk < 1 || rp->topk > rp->K)
        return fail(FOCUS_EINVAL, "topk must be in [1,K] (got %d, K=%d)", rp->topk, rp->K);
    if (rp->dtype != FOCUS_F32 && rp->dtype != FOCUS_BF16 && rp->dtype != FOCUS_F16)
        return fail(FOCUS_EINVAL, "unknown dtype %d", rp->dtype);
    if (rp->sinkhorn_iters < 0) return fail(FOCUS_EINVAL, "sinkhorn_iters must be >= 0");
    if (!(rp->tau > 0.0) || !std::isfinite(rp->tau)) return fail(FOCUS_EINVAL, "tau must be finite and > 0");
    if (rp->d_model % 8 != 0) return fail(FOCUS_EUNSUPPORTED, "d_model %d is not a multiple of 8", rp->d_model);
    if (rp->d_g != 4 && rp->d_g != 8 && rp->d_g != 16 && rp->d_g != 32 && rp->d_g != 64)
        return fail(FOCUS_EUNSUPPORTED, "d_g %d is not built (4, 8, 16, 32 or 64)", rp->d_g);
    if (rp->n > (1 << 24)) return fail(FOCUS_EUNSUPPORTED, "n above 2^24 is not built");
    if (rp->B > 65535) return fail(FOCUS_EUNSUPPORTED, "B above 65535 is not built");
    if (rp->sinkhorn_iters > 1000) return fail(FOCUS_EUNSUPPORTED, "more than 1000 Sinkhorn rounds is not built");
    memset(R, 0, sizeof(*R));
    R->B = rp->B; R->n = rp->n; R->dm = rp->d_model; R->dg = rp->d_g; R->K = rp->K; R->topk = rp->topk;
    R->dtype = rp->dtype; R->iters = rp->sinkhorn_iters; R->tau = rp->tau;
    R->nproj = (rp->n + 63) / 64;
    R->nsink = std::min(256, (rp->n + 255) / 256);
    R->sink_tokens = (rp->n + R->nsink - 1) / R->nsink;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = align256(off + bytes); return o; };
    R->off_w64 = take((size_t)rp->d_model * rp->d_g * 8);
    R->off_c64 = take((size_t)rp->K * rp->d_g * 8);
    R->off_S = take((size_t)rp->B * rp->n * rp->K * 8);
    R->off_maxpart = take((size_t)rp->B * R->nproj * 8);
    R->off_smax = take((size_t)rp->B * 8);
    R->off_colpart = take((size_t)2 * rp->B * R->nsink * 32 * 8);
    R->total = off;
    return FOCUS_OK;
}

// Validates params for the incremental path (p->n is the capacity of the caches) and lays out its state.
focus_status make_decode_layout(const focus_params* p, focus::DecodeLayout* L, focus::HeadMap* hm)
{
    using namespace focus;
    if (!p) return fail(FOCUS_EINVAL, "params is NULL");
    if (p->B < 1 || p->Hq < 1 || p->Hkv < 1 || p->n < 1)
        return fail(FOCUS_EINVAL, "B, Hq, Hkv, n must be >= 1 (got %d %d %d %d)", p->B, p->Hq, p->Hkv, p->n);
    if (p->dtype != FOCUS_F32 && p->dtype != FOCUS_BF16 && p->dtype != FOCUS_F16) return fail(FOCUS_EINVAL, "unknown dtype %d", p->dtype);
    if (p->K < 1 || p->K > 32) return fail(FOCUS_EINVAL, "K must be in [1,32] (got %d)", p->K);
    if (p->topk < 1 || p->topk > p->K) return fail(FOCUS_EINVAL, "topk must be in [1,K] (got %d, K=%d)", p->topk, p->K);
    if (p->window < 1) return fail(FOCUS_EINVAL, "window must be >= 1 (got %d)", p->window);
    if (!(p->scale >= 0.0f) || !std::isfinite(p->scale)) return fail(FOCUS_EINVAL, "scale must be finite and >= 0");
    if (!(p->softcap >= 0.0f) || !std::isfinite(p->softcap)) return fail(FOCUS_EINVAL, "softcap must be finite and >= 0");
    if (p->head_map) {
        for (int h = 0; h < p->Hq; ++h)
            if (p->head_map[h] < 0 || p->head_map[h] >= p->Hkv)
                return fail(FOCUS_EINVAL, "head_map[%d]=%d is outside [0,Hkv)", h, p->head_map[h]);
    } else if (p->Hq % p->Hkv != 0) {
        return fail(FOCUS_EINVAL, "Hq (%d) is not a multiple of Hkv (%d) and no head_map given", p->Hq, p->Hkv);
    }
    if (p->causal != 1) return fail(FOCUS_EUNSUPPORTED, "the incremental path is causal (one new token at the end)");
    if (!contiguous_tensors(p))
        return fail(FOCUS_EUNSUPPORTED, "the incremental path takes contiguous caches and rows (strides must be 0)");
    if (p->d != 64 && p->d != 80 && p->d != 96 && p->d != 128 && p->d != 256)
        return fail(FOCUS_EUNSUPPORTED, "head dim %d is not built (64, 80, 96, 128 or 256)", p->d);
    if (p->Hq > MAX_HQ || p->Hkv > MAX_HQ) return fail(FOCUS_EUNSUPPORTED, "more than %d heads is not built", MAX_HQ);
    if (p->n > (1 << 24)) return fail(FOCUS_EUNSUPPORTED, "n above 2^24 is not built");
    if ((int64_t)p->B * p->Hq > 65535 || (int64_t)p->B * p->Hkv > 65535)
        return fail(FOCUS_EUNSUPPORTED, "B*H above 65535 is not built");
    memset(L, 0, sizeof(*L));
    L->B = p->B; L->Hq = p->Hq; L->Hkv = p->Hkv; L->n = p->n; L->d = p->d;
    L->K = p->K; L->topk = p->topk; L->window = p->window; L->dtype = p->dtype;
    L->scale = (p->scale > 0.0f) ? p->scale : (float)(1.0 / std::sqrt((double)p->d));
    L->softcap = p->softcap;
    // longest key sequence a step walks: n entries (the group lists are used only while they are shorter than
    // the range of positions below the window)
    L->max_chunks = (p->n + DEC_CHUNK - 1) / DEC_CHUNK;
    L->max_parts = std::min((p->n + DEC_CHUNK_SHORT - 1) / DEC_CHUNK_SHORT, DEC_MAX_PARTS);
    for (int h = 0; h < p->Hq; ++h)
        hm->kv[h] = (uint8_t)(p->head_map ? p->head_map[h] : h / (p->Hq / p->Hkv));
    const size_t BHq = (size_t)p->B * p->Hq, BHk = (size_t)p->B * p->Hkv, n = (size_t)p->n;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = align256(off + bytes); return o; };
    L->off_mk = take(BHk * n * 4);
    L->off_lists = take(BHk * (size_t)p->K * n * 4);
    L->off_counts = take(BHk * (size_t)p->K * 4);
    L->off_wp = take(BHk * (size_t)p->K * 4);
    L->off_mq = take(BHq * 4);
    L->off_part = take(BHq * (size_t)L->max_parts * (size_t)(p->d + 4) * 4);
    L->total = off;
    return FOCUS_OK;
}

// The embedded local layout of a two-pass problem: every token in one class, position order (the bucketing with a
// constant membership, as the soft gate uses it), with its own class-ordered -- here: position-ordered -- key copy.
hipError_t assign_local_layout(const focus_params* p, const focus::Layout& L, const void* k, char* ws, hipStream_t st)
{
    if (!L.two_pass) return hipSuccess;
    focus::Layout L2;
    focus::HeadMap hm2;
    if (make_layout(p, &L2, &hm2, false, true) != FOCUS_OK) return hipErrorInvalidValue;
    return focus::launch_assign_tokens(L2, nullptr, k, ws + L.off_local, nullptr, st);
}

}  // namespace

extern "C" {

focus_status focus_workspace_size(const focus_params* p, size_t* bytes)
{
    if (!bytes) return fail(FOCUS_EINVAL, "bytes is NULL");
    focus::Layout L;
    focus::HeadMap hm;
    focus_status st = make_layout(p, &L, &hm);
    if (st != FOCUS_OK) return st;
    *bytes = L.total;
    return FOCUS_OK;
}

focus_status focus_assign(const focus_params* p, const void* q, const void* k, const float* centroids,
                          void* workspace, size_t workspace_bytes, void* stream)
{
    focus::Layout L;
    focus::HeadMap hm;
    focus_status st = make_layout(p, &L, &hm);
    if (st != FOCUS_OK) return st;
    if (!q || !k || !centroids) return fail(FOCUS_EINVAL, "q, k and centroids must not be NULL");
    if (misaligned16(q) || misaligned16(k) || misaligned16(centroids))
        return fail(FOCUS_EINVAL, "q, k and centroids must be 16-byte aligned");
    st = check_ws(L, workspace, workspace_bytes);
    if (st != FOCUS_OK) return st;
    hipError_t e = focus::launch_assign(L, hm, q, k, centroids, (char*)workspace, (hipStream_t)stream);
    if (e == hipSuccess) e = assign_local_layout(p, L, k, (char*)workspace, (hipStream_t)stream);
    if (e != hipSuccess) return fail(FOCUS_EHIP, "focus_assign: %s", hipGetErrorString(e));
    return FOCUS_OK;
}

namespace {

// one launch of the attention kernels over the whole mask (pair_set 0) or one of its two disjoint parts
focus_status attn_launch(const focus_params* p, int pair_set, const void* q, const void* k, const void* v,
                         void* workspace, size_t workspace_bytes, void* out, float* lse, int32_t* row_pairs,
                         void* stream, const char* who, bool force_vector = false)
{
    focus::Layout L;
    focus::HeadMap hm;
    focus_status st = make_layout(p, &L, &hm);
    if (st != FOCUS_OK) return st;
    if (pair_set < 0 || pair_set > 2) return fail(FOCUS_EINVAL, "pair_set must be 0, 1 or 2 (got %d)", pair_set);
    if (pair_set != 0 && p->window >= p->n && 2 * p->topk <= p->K)
        return fail(FOCUS_EUNSUPPORTED, "the two-set decomposition is not built for window >= n "
                                        "(every causal pair is local: one launch over the whole mask is the answer)");
    if (!q || !k || !v || !out) return fail(FOCUS_EINVAL, "q, k, v and out must not be NULL");
    if (misaligned16(q) || misaligned16(k) || misaligned16(v) || misaligned16(out))
        return fail(FOCUS_EINVAL, "q, k, v and out must be 16-byte aligned");
    if (out == q || out == k || out == v) return fail(FOCUS_EINVAL, "out must not alias an input");
    st = check_ws(L, workspace, workspace_bytes);
    if (st != FOCUS_OK) return st;
    L.pair_set = pair_set;
    hipError_t e;
    if (L.two_pass && pair_set == 0 && !force_vector) {
        // Pass 1: every pair inside the window (whatever the groups) over position-ordered 128-row tiles: the
        // band is then covered by tiles of consecutive positions, almost none of them masked.  Pass 2: the pairs
        // outside the window that share a group, over the class-ordered tiles; its epilogue merges the two partial
        // softmaxes of a row through their log-sum-exp (App. D's merge), so each allowed pair still counts once.
        focus::Layout L2;
        focus::HeadMap hm2;
        st = make_layout(p, &L2, &hm2, false, true);
        if (st != FOCUS_OK) return st;
        float* lse1 = lse ? lse : (float*)((char*)workspace + L.off_lse1);
        e = focus::launch_attn_mfma(L2, hm2, q, k, v, nullptr, (char*)workspace + L.off_local, out, lse1, row_pairs,
                                    (hipStream_t)stream);
        if (e == hipSuccess) {
            L.pair_set = 3;
            L.merge_prev = 1;
            e = focus::launch_attn_mfma(L, hm, q, k, v, nullptr, (char*)workspace, out, lse1, row_pairs, (hipStream_t)stream);
        }
    } else if (L.dtype != FOCUS_F32 && !force_vector)
        e = focus::launch_attn_mfma(L, hm, q, k, v, nullptr, (char*)workspace, out, lse, row_pairs, (hipStream_t)stream);
    else
        e = focus::launch_attn_simple(L, hm, q, k, v, nullptr, (char*)workspace, out, lse, row_pairs, (hipStream_t)stream);
    if (e != hipSuccess) return fail(FOCUS_EHIP, "%s: %s", who, hipGetErrorString(e));
    return FOCUS_OK;
}

}  // namespace

focus_status focus_attn_fwd(const focus_params* p, const void* q, const void* k, const void* v,
                            void* workspace, size_t workspace_bytes, void* out, float* lse,
                            int32_t* row_pairs, void* stream)
{
    return attn_launch(p, 0, q, k, v, workspace, workspace_bytes, out, lse, row_pairs, stream, "focus_attn_fwd");
}

focus_status focus_attn_fwd_set(const focus_params* p, int32_t pair_set, const void* q, const void* k, const void* v,
                                void* workspace, size_t workspace_bytes, void* out, float* lse, int32_t* row_pairs,
                                void* stream)
{
    return attn_launch(p, pair_set, q, k, v, workspace, workspace_bytes, out, lse, row_pairs, stream,
                       "focus_attn_fwd_set");
}

focus_status focus_attn_merge(int64_t rows, int32_t d, int32_t dtype, const void* out_a, const float* lse_a,
                              const void* out_b, const float* lse_b, void* out, float* lse, void* stream)
{
    if (rows < 0 || d < 8 || d % 8 != 0) return fail(FOCUS_EINVAL, "rows must be >= 0 and d a positive multiple of 8");
    if (dtype != FOCUS_F32 && dtype != FOCUS_BF16 && dtype != FOCUS_F16) return fail(FOCUS_EINVAL, "unknown dtype %d", dtype);
    if (!out_a || !lse_a || !out_b || !lse_b || !out) return fail(FOCUS_EINVAL, "partial outputs, their lse and out must not be NULL");
    if (misaligned16(out_a) || misaligned16(out_b) || misaligned16(out))
        return fail(FOCUS_EINVAL, "out_a, out_b and out must be 16-byte aligned");
    if (rows == 0) return FOCUS_OK;
    hipError_t e = focus::launch_attn_merge((size_t)rows, d, dtype, out_a, lse_a, out_b, lse_b, out, lse,
                                            (hipStream_t)stream);
    if (e != hipSuccess) return fail(FOCUS_EHIP, "focus_attn_merge: %s", hipGetErrorString(e));
    return FOCUS_OK;
}

focus_status focus_attn_fwd_two_call(const focus_params* p, const void* q, const void* k, const void* v,
                                     void* workspace, size_t workspace_bytes, void* out, float* lse, void* part_out,
                                     float* part_lse, void* stream)
{
    if (!p) return fail(FOCUS_EINVAL, "params is NULL");
    if (!part_out || !part_lse) return fail(FOCUS_EINVAL, "part_out and part_lse must not be NULL");
    if (!contiguous_tensors(p))
        return fail(FOCUS_EUNSUPPORTED, "focus_attn_fwd_two_call takes contiguous tensors (use focus_attn_fwd_set and "
                                        "focus_attn_merge on contiguous partial outputs, or the fused focus_attn_fwd)");
    if (misaligned16(part_out)) return fail(FOCUS_EINVAL, "part_out must be 16-byte aligned");
    if (!out) return fail(FOCUS_EINVAL, "out must not be NULL");
    if (misaligned16(out)) return fail(FOCUS_EINVAL, "out must be 16-byte aligned");
    if (out == q || out == k || out == v) return fail(FOCUS_EINVAL, "out must not alias an input");
    const size_t rows = (size_t)p->B * (size_t)p->Hq * (size_t)p->n;
    const size_t elem = (p->dtype == FOCUS_F32) ? 4 : 2;
    char* oa = (char*)part_out;
    char* ob = oa + rows * (size_t)p->d * elem;
    float* la = part_lse;
    float* lb = part_lse + rows;
    focus_status st = attn_launch(p, 1, q, k, v, workspace, workspace_bytes, oa, la, nullptr, stream,
                                  "focus_attn_fwd_two_call (set A)");
    if (st != FOCUS_OK) return st;
    st = attn_launch(p, 2, q, k, v, workspace, workspace_bytes, ob, lb, nullptr, stream,
                     "focus_attn_fwd_two_call (set B)");
    if (st != FOCUS_OK) return st;
    return focus_attn_merge((int64_t)rows, p->d, p->dtype, oa, la, ob, lb, out, lse, stream);
}

// Same contract and the same argument checks as focus_attn_fwd, but always through the fp32 vector kernel
// (no matrix cores): the on-device cross-check of the MFMA kernel at sizes the CPU oracle cannot cover in full.
focus_status focus_attn_fwd_vector(const focus_params* p, const void* q, const void* k, const void* v,
                                   void* workspace, size_t workspace_bytes, void* out, float* lse,
                                   int32_t* row_pairs, void* stream)
{
    return attn_launch(p, 0, q, k, v, workspace, workspace_bytes, out, lse, row_pairs, stream,
                       "focus_attn_fwd_vector", true);
}

namespace {

focus_status soft_checks(const focus_params* p)
{
    if (p && p->causal != 1) return fail(FOCUS_EUNSUPPORTED, "the soft-gated attention is causal (Sec. 2 Eq. 2)");
    if (p && p->softcap != 0.0f) return fail(FOCUS_EUNSUPPORTED, "the soft-gated attention takes no softcap");
    return FOCUS_OK;
}

focus_status soft_launch(const focus_params* p, float lambda, const float* g, const void* q, const void* k,
                         const void* v, void* workspace, size_t workspace_bytes, void* out, float* lse, void* stream,
                         bool vector)
{
    focus::Layout L;
    focus::HeadMap hm;
    focus_status st = soft_checks(p);
    if (st != FOCUS_OK) return st;
    st = make_layout(p, &L, &hm, true);
    if (st != FOCUS_OK) return st;
    if (!std::isfinite(lambda)) return fail(FOCUS_EINVAL, "lambda must be finite");
    if (!g || !q || !k || !v || !out) return fail(FOCUS_EINVAL, "g, q, k, v and out must not be NULL");
    if (misaligned16(q) || misaligned16(k) || misaligned16(v) || misaligned16(out))
        return fail(FOCUS_EINVAL, "q, k, v and out must be 16-byte aligned");
    if (out == q || out == k || out == v) return fail(FOCUS_EINVAL, "out must not alias an input");
    st = check_ws(L, workspace, workspace_bytes);
    if (st != FOCUS_OK) return st;
    L.gate_slope = (float)(-(double)lambda * 1.4426950408889634);
    // head dim 256 in a 16-bit type: the gate's accumulators and operands do not fit the register file next to
    // 512-byte key rows, so that shape goes through the vector kernel (correct, slow)
    if (p->d == 256) vector = true;
    hipStream_t s = (hipStream_t)stream;
    // one class holding every token, in position order: the bucketing with a constant membership
    hipError_t e = focus::launch_assign_tokens(L, nullptr, k, (char*)workspace, nullptr, s);
    if (e == hipSuccess && L.dtype != FOCUS_F32 && !vector) e = focus::launch_soft_gather_g(L, g, (char*)workspace, s);
    if (e == hipSuccess) {
        if (L.dtype != FOCUS_F32 && !vector)
            e = focus::launch_attn_mfma(L, hm, q, k, v, g, (char*)workspace, out, lse, nullptr, s);
        else
            e = focus::launch_attn_simple(L, hm, q, k, v, g, (char*)workspace, out, lse, nullptr, s);
    }
    if (e != hipSuccess) return fail(FOCUS_EHIP, "focus_attn_soft_fwd: %s", hipGetErrorString(e));
    return FOCUS_OK;
}

}  // namespace

focus_status focus_soft_workspace_size(const focus_params* p, size_t* bytes)
{
    if (!bytes) return fail(FOCUS_EINVAL, "bytes is NULL");
    focus::Layout L;
    focus::HeadMap hm;
    focus_status st = soft_checks(p);
    if (st != FOCUS_OK) return st;
    st = make_layout(p, &L, &hm, true);
    if (st != FOCUS_OK) return st;
    *bytes = L.total;
    return FOCUS_OK;
}

focus_status focus_attn_soft_fwd(const focus_params* p, float lambda, const float* g, const void* q, const void* k,
                                 const void* v, void* workspace, size_t workspace_bytes, void* out, float* lse,
                                 void* stream)
{
    return soft_launch(p, lambda, g, q, k, v, workspace, workspace_bytes, out, lse, stream, false);
}

// The same through the fp32 vector kernel (cross-check of the MFMA kernel in tests).
focus_status focus_attn_soft_fwd_vector(const focus_params* p, float lambda, const float* g, const void* q,
                                        const void* k, const void* v, void* workspace, size_t workspace_bytes,
                                        void* out, float* lse, void* stream)
{
    return soft_launch(p, lambda, g, q, k, v, workspace, workspace_bytes, out, lse, stream, true);
}

focus_status focus_route_workspace_size(const focus_route_params* rp, size_t* bytes)
{
    if (!bytes) return fail(FOCUS_EINVAL, "bytes is NULL");
    focus::RouteLayout R;
    focus_status st = make_route_layout(rp, &R);
    if (st != FOCUS_OK) return st;
    *bytes = R.total;
    return FOCUS_OK;
}

focus_status focus_route(const focus_route_params* rp, const void* hidden, const float* w_g, const float* centroids,
                         void* route_workspace, size_t workspace_bytes, uint32_t* token_masks, double* soft,
                         void* stream)
{
    focus::RouteLayout R;
    focus_status st = make_route_layout(rp, &R);
    if (st != FOCUS_OK) return st;
    if (!hidden || !w_g || !centroids || !token_masks)
        return fail(FOCUS_EINVAL, "hidden, w_g, centroids and token_masks must not be NULL");
    if (misaligned16(hidden)) return fail(FOCUS_EINVAL, "hidden must be 16-byte aligned");
    if (!route_workspace) return fail(FOCUS_EINVAL, "route workspace is NULL");
    if (((uintptr_t)route_workspace & 255) != 0) return fail(FOCUS_EWORKSPACE, "route workspace is not 256-byte aligned");
    if (workspace_bytes < R.total)
        return fail(FOCUS_EWORKSPACE, "route workspace has %zu bytes, %zu needed", workspace_bytes, R.total);
    hipError_t e = focus::launch_route(R, hidden, w_g, centroids, (char*)route_workspace, token_masks, soft,
                                       (hipStream_t)stream);
    if (e != hipSuccess) return fail(FOCUS_EHIP, "focus_route: %s", hipGetErrorString(e));
    return FOCUS_OK;
}

focus_status focus_route_noalloc(const focus_route_params* rp, const void* hidden, const float* w_g,
                                 const float* centroids, uint32_t* token_masks, double* soft, void* stream)
{
    focus::RouteLayout R;
    focus_status st = make_route_layout(rp, &R);
    if (st != FOCUS_OK) return st;
    if (!hidden || !w_g || !centroids || !token_masks)
        return fail(FOCUS_EINVAL, "hidden, w_g, centroids and token_masks must not be NULL");
    if (misaligned16(hidden)) return fail(FOCUS_EINVAL, "hidden must be 16-byte aligned");
    if (R.total > focus::ROUTE_STATIC_SCRATCH_BYTES)
        return fail(FOCUS_EWORKSPACE, "focus_route_noalloc: this problem needs %zu bytes of scratch, the library's "
                                      "static buffer holds %zu (use focus_route with a workspace of your own)",
                    R.total, focus::ROUTE_STATIC_SCRATCH_BYTES);
    char* ws = nullptr;
    hipError_t e = focus::route_static_scratch(&ws);
    if (e != hipSuccess) return fail(FOCUS_EHIP, "focus_route_noalloc: static scratch: %s", hipGetErrorString(e));
    // every part of the scratch the kernels read is written earlier in the same call: nothing needs clearing
    e = focus::launch_route(R, hidden, w_g, centroids, ws, token_masks, soft, (hipStream_t)stream);
    if (e != hipSuccess) return fail(FOCUS_EHIP, "focus_route_noalloc: %s", hipGetErrorString(e));
    return FOCUS_OK;
}

focus_status focus_assign_tokens(const focus_params* p, const uint32_t* token_masks, const void* k, void* workspace,
                                 size_t workspace_bytes, int32_t* invalid_count, void* stream)
{
    focus::Layout L;
    focus::HeadMap hm;
    focus_status st = make_layout(p, &L, &hm);
    if (st != FOCUS_OK) return st;
    if (!token_masks || !k) return fail(FOCUS_EINVAL, "token_masks and k must not be NULL");
    if (misaligned16(k)) return fail(FOCUS_EINVAL, "k must be 16-byte aligned");
    st = check_ws(L, workspace, workspace_bytes);
    if (st != FOCUS_OK) return st;
    hipError_t e = focus::launch_assign_tokens(L, token_masks, k, (char*)workspace, invalid_count, (hipStream_t)stream);
    if (e == hipSuccess) e = assign_local_layout(p, L, k, (char*)workspace, (hipStream_t)stream);
    if (e != hipSuccess) return fail(FOCUS_EHIP, "focus_assign_tokens: %s", hipGetErrorString(e));
    return FOCUS_OK;
}

focus_status focus_decode_state_size(const focus_params* p, size_t* bytes)
{
    if (!bytes) return fail(FOCUS_EINVAL, "bytes is NULL");
    focus::DecodeLayout L;
    focus::HeadMap hm;
    focus_status st = make_decode_layout(p, &L, &hm);
    if (st != FOCUS_OK) return st;
    *bytes = L.total;
    return FOCUS_OK;
}

namespace {

focus_status decode_prefill_common(const focus_params* p, int32_t n_ctx, const void* k_cache, const float* centroids,
                                   const uint32_t* token_masks, void* state, size_t state_bytes, void* stream,
                                   const char* who)
{
    focus::DecodeLayout L;
    focus::HeadMap hm;
    focus_status st = make_decode_layout(p, &L, &hm);
    if (st != FOCUS_OK) return st;
    if (n_ctx < 0 || n_ctx > p->n) return fail(FOCUS_EINVAL, "n_ctx must be in [0, n] (got %d, n=%d)", n_ctx, p->n);
    if (!token_masks && (!k_cache || !centroids)) return fail(FOCUS_EINVAL, "k_cache and centroids must not be NULL");
    if (!token_masks && misaligned16(k_cache)) return fail(FOCUS_EINVAL, "k_cache must be 16-byte aligned");
    if (!state) return fail(FOCUS_EINVAL, "state is NULL");
    if (((uintptr_t)state & 255) != 0) return fail(FOCUS_EWORKSPACE, "state is not 256-byte aligned");
    if (state_bytes < L.total) return fail(FOCUS_EWORKSPACE, "state has %zu bytes, %zu needed", state_bytes, L.total);
    hipError_t e = focus::launch_decode_prefill(L, n_ctx, k_cache, centroids, token_masks, (char*)state, (hipStream_t)stream);
    if (e != hipSuccess) return fail(FOCUS_EHIP, "%s: %s", who, hipGetErrorString(e));
    return FOCUS_OK;
}

focus_status decode_step_common(const focus_params* p, int32_t pos, const int32_t* pos_dev, const void* q_new,
                                const void* k_new, const void* v_new, const float* centroids,
                                const uint32_t* token_mask, void* k_cache, void* v_cache, void* state,
                                size_t state_bytes, void* out, float* lse, int32_t* row_pairs, void* stream,
                                const char* who)
{
    focus::DecodeLayout L;
    focus::HeadMap hm;
    focus_status st = make_decode_layout(p, &L, &hm);
    if (st != FOCUS_OK) return st;
    if (!pos_dev && (pos < 0 || pos >= p->n)) return fail(FOCUS_EINVAL, "pos must be in [0, n) (got %d, n=%d)", pos, p->n);
    if (!q_new || !k_new || !v_new || (!centroids && !token_mask) || !k_cache || !v_cache || !out)
        return fail(FOCUS_EINVAL, "q_new, k_new, v_new, centroids (or the token mask), k_cache, v_cache and out must not be NULL");
    if (misaligned16(q_new) || misaligned16(k_new) || misaligned16(v_new) || misaligned16(k_cache) ||
        misaligned16(v_cache) || misaligned16(out))
        return fail(FOCUS_EINVAL, "q_new, k_new, v_new, k_cache, v_cache and out must be 16-byte aligned");
    if (!state) return fail(FOCUS_EINVAL, "state is NULL");
    if (((uintptr_t)state & 255) != 0) return fail(FOCUS_EWORKSPACE, "state is not 256-byte aligned");
    if (state_bytes < L.total) return fail(FOCUS_EWORKSPACE, "state has %zu bytes, %zu needed", state_bytes, L.total);
    hipError_t e = focus::launch_decode_step(L, hm, pos, pos_dev, q_new, k_new, v_new, centroids, token_mask, k_cache,
                                             v_cache, (char*)state, out, lse, row_pairs, (hipStream_t)stream);
    if (e != hipSuccess) return fail(FOCUS_EHIP, "%s: %s", who, hipGetErrorString(e));
    return FOCUS_OK;
}

}  // namespace

focus_status focus_decode_prefill(const focus_params* p, int32_t n_ctx, const void* k_cache, const float* centroids,
                                  void* state, size_t state_bytes, void* stream)
{
    return decode_prefill_common(p, n_ctx, k_cache, centroids, nullptr, state, state_bytes, stream, "focus_decode_prefill");
}

focus_status focus_decode_prefill_tokens(const focus_params* p, int32_t n_ctx, const uint32_t* token_masks, void* state,
                                         size_t state_bytes, void* stream)
{
    if (!token_masks && n_ctx > 0) return fail(FOCUS_EINVAL, "token_masks is NULL");
    static const uint32_t none = 0;                  // n_ctx = 0: nothing is read, any non-NULL pointer selects the path
    return decode_prefill_common(p, n_ctx, nullptr, nullptr, token_masks ? token_masks : &none, state, state_bytes, stream,
                                 "focus_decode_prefill_tokens");
}

focus_status focus_decode_step(const focus_params* p, int32_t pos, const void* q_new, const void* k_new,
                               const void* v_new, const float* centroids, void* k_cache, void* v_cache, void* state,
                               size_t state_bytes, void* out, float* lse, int32_t* row_pairs, void* stream)
{
    if (!centroids) return fail(FOCUS_EINVAL, "centroids is NULL");
    return decode_step_common(p, pos, nullptr, q_new, k_new, v_new, centroids, nullptr, k_cache, v_cache, state,
                              state_bytes, out, lse, row_pairs, stream, "focus_decode_step");
}

focus_status focus_decode_step_at(const focus_params* p, const int32_t* pos_dev, const void* q_new, const void* k_new,
                                  const void* v_new, const float* centroids, void* k_cache, void* v_cache,
                                  void* state, size_t state_bytes, void* out, float* lse, int32_t* row_pairs,
                                  void* stream)
{
    if (!pos_dev) return fail(FOCUS_EINVAL, "pos_dev is NULL");
    if (!centroids) return fail(FOCUS_EINVAL, "centroids is NULL");
    return decode_step_common(p, 0, pos_dev, q_new, k_new, v_new, centroids, nullptr, k_cache, v_cache, state,
                              state_bytes, out, lse, row_pairs, stream, "focus_decode_step_at");
}

focus_status focus_decode_step_tokens(const focus_params* p, int32_t pos, const uint32_t* token_mask, const void* q_new,
                                      const void* k_new, const void* v_new, void* k_cache, void* v_cache, void* state,
                                      size_t state_bytes, void* out, float* lse, int32_t* row_pairs, void* stream)
{
    if (!token_mask) return fail(FOCUS_EINVAL, "token_mask is NULL");
    return decode_step_common(p, pos, nullptr, q_new, k_new, v_new, nullptr, token_mask, k_cache, v_cache, state,
                              state_bytes, out, lse, row_pairs, stream, "focus_decode_step_tokens");
}

focus_status focus_decode_state_views(const focus_params* p, void* state, const uint32_t** mk, const int32_t** lists,
                                      const int32_t** counts, const uint32_t** mq)
{
    focus::DecodeLayout L;
    focus::HeadMap hm;
    focus_status st = make_decode_layout(p, &L, &hm);
    if (st != FOCUS_OK) return st;
    if (!state) return fail(FOCUS_EINVAL, "state is NULL");
    char* s = (char*)state;
    if (mk) *mk = (const uint32_t*)(s + L.off_mk);
    if (lists) *lists = (const int32_t*)(s + L.off_lists);
    if (counts) *counts = (const int32_t*)(s + L.off_counts);
    if (mq) *mq = (const uint32_t*)(s + L.off_mq);
    return FOCUS_OK;
}

focus_status focus_workspace_views(const focus_params* p, void* workspace, const uint32_t** mq,
                                   const uint32_t** mk, const int32_t** q_group_counts,
                                   const int32_t** k_group_counts, const int32_t** q_group_lists,
                                   const int32_t** k_group_lists)
{
    focus::Layout L;
    focus::HeadMap hm;
    focus_status st = make_layout(p, &L, &hm);
    if (st != FOCUS_OK) return st;
    if (!workspace) return fail(FOCUS_EINVAL, "workspace is NULL");
    char* ws = (char*)workspace;
    if (mq) *mq = (const uint32_t*)(ws + L.off_mq);
    if (mk) *mk = (const uint32_t*)(ws + L.off_mk);
    if (q_group_counts) *q_group_counts = (const int32_t*)(ws + L.off_qgc);
    if (k_group_counts) *k_group_counts = (const int32_t*)(ws + L.off_kgc);
    if (q_group_lists) *q_group_lists = (const int32_t*)(ws + L.off_qgl);
    if (k_group_lists) *k_group_lists = (const int32_t*)(ws + L.off_kgl);
    return FOCUS_OK;
}

const char* focus_last_error(void) { return g_err; }

int focus_version(void) { return 100; }

#ifndef FOCUS_BUILD_ID
#define FOCUS_BUILD_ID "unknown"
#endif
const char* focus_build_id(void) { return FOCUS_BUILD_ID; }

}  // extern "C"
