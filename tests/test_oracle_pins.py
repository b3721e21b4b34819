"""Pins of the CPU oracle against things other than itself (no GPU needed).

P1 brute force on tiny problems; P2-P5 reductions to dense attention checked
against torch's scaled_dot_product_attention in fp64; P6 probability rows;
P7/P8 pair-count closed forms; P9 the paper's disjoint two-set decomposition
with its log-sum-exp merge (App. D); P10 softcap limits; P11 expected retained
fraction; P12 metamorphic relations; plus score/top-k/list/GQA pins.
"""
import itertools
import math
import os

import numpy as np
import pytest
import torch

from oracle import focus_oracle as fo
from tests import brute

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rand_problem(seed, B, Hq, Hkv, n, d, K, dtype="f32"):
    rng = np.random.default_rng(seed)
    q = rng.standard_normal((B, Hq, n, d)).astype(np.float32)
    k = rng.standard_normal((B, Hkv, n, d)).astype(np.float32)
    v = rng.standard_normal((B, Hkv, n, d)).astype(np.float32)
    c = rng.standard_normal((Hkv, K, d))
    c = (c / np.linalg.norm(c, axis=-1, keepdims=True)).astype(np.float32)
    if dtype == "bf16":
        q, k, v = (torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
                   for x in (q, k, v))
    return q, k, v, c


def run_oracle(pb, q, k, v, c, rows=None, want_probs=False):
    mq = fo.membership(pb, q, c, True)
    mk = fo.membership(pb, k, c, False)
    res = fo.attn_rows(pb, q, k, v, mq, mk, rows=rows, want_probs=want_probs)
    return (mq, mk) + tuple(res)


def sdpa64(q, k, v, causal, Hq, Hkv, head_map=None, scale=None):
    q, k, v = (torch.from_numpy(brute.as_f64(x)) for x in (q, k, v))
    if head_map is None:
        head_map = [h // (Hq // Hkv) for h in range(Hq)]
    k = k[:, head_map]
    v = v[:, head_map]
    return torch.nn.functional.scaled_dot_product_attention(
        q, k, v, is_causal=causal, scale=scale).numpy()


# ---------------------------------------------------------------- P1 brute force
TINY = []
for n_, d_, K_ in [(1, 1, 1), (2, 2, 2), (3, 1, 3), (5, 4, 4), (8, 2, 3), (17, 4, 4)]:
    for topk_ in range(1, K_ + 1):
        for w_ in sorted({1, 2, n_, n_ + 3}):
            TINY.append((n_, d_, K_, topk_, w_))


@pytest.mark.parametrize("n,d,K,topk,w", TINY)
@pytest.mark.parametrize("causal", [True, False])
def test_p1_brute_force(n, d, K, topk, w, causal):
    q, k, v, c = rand_problem(100 + n * 7 + d, 1, 2, 1, n, d, K)
    pb = fo.Problem(1, 2, 1, n, d, K, topk, w, causal=causal)
    mq, mk, out, lse, pairs = run_oracle(pb, q, k, v, c)
    bo, bl, bp, iq, ik = brute.attention(q, k, v, c, topk, w, causal=causal)
    want_mq = np.array([[[brute.ids_to_mask(iq[0][h][i]) for i in range(n)] for h in range(2)]])
    want_mk = np.array([[[brute.ids_to_mask(ik[0][0][j]) for j in range(n)]]])
    assert np.array_equal(mq, want_mq)
    assert np.array_equal(mk, want_mk)
    assert np.array_equal(pairs.reshape(1, 2, n), bp)
    np.testing.assert_allclose(out.reshape(1, 2, n, d), bo, atol=1e-12, rtol=0)
    np.testing.assert_allclose(lse.reshape(1, 2, n), bl, atol=1e-12, rtol=0)


def test_p1_brute_force_bf16_gqa_softcap():
    q, k, v, c = rand_problem(7, 2, 4, 2, 12, 4, 4, dtype="bf16")
    hm = np.array([1, 0, 0, 1], dtype=np.int32)
    pb = fo.Problem(2, 4, 2, 12, 4, 4, 2, 3, dtype="bf16", softcap=0.7, scale=0.9, head_map=hm)
    mq, mk, out, lse, pairs = run_oracle(pb, q, k, v, c)
    bo, bl, bp, iq, ik = brute.attention(q, k, v, c, 2, 3, head_map=list(hm), scale=0.9, softcap=0.7)
    assert np.array_equal(pairs.reshape(2, 4, 12), bp)
    np.testing.assert_allclose(out.reshape(2, 4, 12, 4), bo, atol=1e-12, rtol=0)
    np.testing.assert_allclose(lse.reshape(2, 4, 12), bl, atol=1e-12, rtol=0)


# ------------------------------------------------- P2-P5 reductions to dense attention
@pytest.mark.parametrize("K,topk,w,causal", [
    (1, 1, 3, True),        # P2: one group
    (4, 2, 64, True),       # P3: window covers the sequence
    (4, 2, 200, True),      # P3: window beyond the sequence
    (4, 4, 5, True),        # P4: every group kept
    (4, 4, 5, False),       # P4 non-causal: full bidirectional attention
    (4, 3, 5, True),        # P5: 2k > K, any two sets meet (Table 7: k=3 of 4 keeps 100 %)
    (5, 3, 2, True),        # P5
    (8, 5, 1, False),       # P5 non-causal
])
def test_reduces_to_dense_attention(K, topk, w, causal):
    B, Hq, Hkv, n, d = 2, 4, 2, 64, 8
    q, k, v, c = rand_problem(11 + K + topk, B, Hq, Hkv, n, d, K)
    pb = fo.Problem(B, Hq, Hkv, n, d, K, topk, w, causal=causal)
    mq, mk, out, lse, pairs = run_oracle(pb, q, k, v, c)
    want = sdpa64(q, k, v, causal, Hq, Hkv)
    np.testing.assert_allclose(out.reshape(B, Hq, n, d), want, atol=1e-12, rtol=0)
    full = (np.arange(n) + 1) if causal else np.full(n, n)
    assert np.array_equal(pairs.reshape(B, Hq, n), np.broadcast_to(full, (B, Hq, n)))


def test_table7_full_retention_rows():
    """Table 7 prints 100 % pairs retained for k=3 and k=4 at K=4."""
    rows = [l.split() for l in open(os.path.join(GOLDEN, "table7_pairs_retained.txt"))
            if l.strip() and not l.startswith("#")]
    n = 96
    for K, topk, pct in rows:
        K, topk, pct = int(K), int(topk), float(pct)
        if pct != 100.0:
            continue
        q, k, v, c = rand_problem(5, 1, 2, 2, n, 8, K)
        pb = fo.Problem(1, 2, 2, n, 8, K, topk, 1)
        mq = fo.membership(pb, q, c, True)
        mk = fo.membership(pb, k, c, False)
        allowed, _ = fo.pair_counts(pb, mq, mk)
        assert np.all(allowed == n * (n + 1) // 2)


# ---------------------------------------------------------------- P6 probability rows
def test_p6_rows_sum_to_one_and_hull():
    B, Hq, Hkv, n, d, K = 1, 2, 1, 50, 6, 4
    q, k, v, c = rand_problem(3, B, Hq, Hkv, n, d, K)
    pb = fo.Problem(B, Hq, Hkv, n, d, K, 1, 4, softcap=2.0)
    mq, mk, out, lse, pairs, probs = run_oracle(pb, q, k, v, c, want_probs=True)
    np.testing.assert_allclose(probs.sum(axis=1), 1.0, atol=1e-12)
    assert np.array_equal((probs > 0).sum(axis=1), pairs)
    # zero probability exactly where App. D's mask (with sets) forbids the pair
    for r in range(B * Hq * n):
        h, i = (r // n) % Hq, r % n
        for j in range(n):
            ok = j <= i and ((i - j < 4) or (mq[0, h, i] & mk[0, 0, j]) != 0)
            assert (probs[r, j] > 0) == ok
    vv = v.astype(np.float64)[0, 0]
    o = out.reshape(Hq, n, d)
    for h in range(Hq):
        for i in range(n):
            sel = probs[h * n + i] > 0
            assert np.all(o[h, i] <= vv[sel].max(axis=0) + 1e-12)
            assert np.all(o[h, i] >= vv[sel].min(axis=0) - 1e-12)


# ---------------------------------------------------------------- P7 pair counts
@pytest.mark.parametrize("K,topk,w,causal", [(4, 2, 8, True), (4, 1, 1, True), (8, 2, 16, True),
                                             (8, 3, 5, True), (6, 2, 300, True), (4, 2, 8, False),
                                             (3, 1, 40, False)])
def test_p7_closed_form_equals_row_popcounts(K, topk, w, causal):
    B, Hq, Hkv, n, d = 2, 4, 2, 150, 8
    q, k, v, c = rand_problem(21 + K, B, Hq, Hkv, n, d, K)
    pb = fo.Problem(B, Hq, Hkv, n, d, K, topk, w, causal=causal)
    mq, mk, out, lse, pairs = run_oracle(pb, q, k, v, c)
    allowed, gp = fo.pair_counts(pb, mq, mk)
    assert np.array_equal(allowed, pairs.reshape(B, Hq, n).sum(axis=2).astype(np.uint64))
    # independent count straight from the bit masks
    for b in range(B):
        for h in range(Hq):
            hk = h // (Hq // Hkv)
            share = (mq[b, h][:, None] & mk[b, hk][None, :]) != 0
            ii, jj = np.meshgrid(np.arange(n), np.arange(n), indexing="ij")
            rng_ok = (jj <= ii) if causal else np.ones_like(share)
            near = (ii - jj < w) & (jj - ii < w)
            assert allowed[b, h] == int((rng_ok & (near | share)).sum())
            for g in range(K):
                bq = ((mq[b, h] >> g) & 1).astype(bool)
                bk = ((mk[b, hk] >> g) & 1).astype(bool)
                assert gp[b, h, g] == int((rng_ok & bq[:, None] & bk[None, :]).sum())


@pytest.mark.parametrize("n,K,w", [(64, 4, 8), (1000, 8, 33), (257, 4, 300), (100, 3, 1)])
def test_p8_balanced_hard_assignment(n, K, w):
    """g(i) = i mod K for queries and keys, k=1: the n^2/K cost model of Sec. 3.6 made exact."""
    d = K
    eye = np.eye(K, dtype=np.float32)
    x = eye[np.arange(n) % K][None, None]                      # [1,1,n,d]
    c = eye[None]                                              # [1,K,d]
    pb = fo.Problem(1, 1, 1, n, d, K, 1, w)
    mq = fo.membership(pb, x, c, True)
    mk = fo.membership(pb, x, c, False)
    assert np.array_equal(mq[0, 0], (1 << (np.arange(n) % K)).astype(np.uint32))
    allowed, gp = fo.pair_counts(pb, mq, mk)
    same = 0
    for r in range(K):
        cr = len(range(r, n, K))
        same += cr * (cr + 1) // 2
        assert gp[0, 0, r] == cr * (cr + 1) // 2
    ww = min(w, n)
    local = ww * (ww + 1) // 2 + (n - ww) * ww
    both = sum(min(w - 1, i) // K + 1 for i in range(n))       # same residue inside the window
    assert allowed[0, 0] == same + local - both
    # and the cost model: same-group causal pairs ~ n^2 / (2K)
    assert abs(same - n * n / (2 * K)) <= n


# ------------------------------------------------ P9 the paper's two-set decomposition
@pytest.mark.parametrize("symmetric", [True, False])
def test_p9_disjoint_decomposition_merge(symmetric):
    B, Hq, Hkv, n, d, K, w = 1, 2, 2, 40, 8, 4, 5
    q, k, v, c = rand_problem(31, B, Hq, Hkv, n, d, K)
    if symmetric:
        k = q.copy()            # same vector scored -> g(i) is one assignment per token
    pb = fo.Problem(B, Hq, Hkv, n, d, K, 1, w)
    mq, mk, out, lse, pairs = run_oracle(pb, q, k, v, c)
    if symmetric:
        assert np.array_equal(mq, mk)
    out = out.reshape(B, Hq, n, d)
    q64, k64, v64 = (x.astype(np.float64) for x in (q, k, v))
    ii, jj = np.meshgrid(np.arange(n), np.arange(n), indexing="ij")
    for h in range(Hq):
        same = (mq[0, h][:, None] & mk[0, h][None, :]) != 0
        A = (jj <= ii) & same                                   # same-group causal
        Bset = (jj <= ii) & (ii - jj < w) & ~same               # cross-group local
        assert not np.any(A & Bset)
        logits = (q64[0, h] @ k64[0, h].T) / math.sqrt(d)

        def part(mask):
            x = np.where(mask, logits, -np.inf)
            m = x.max(axis=1, keepdims=True)
            m = np.where(np.isfinite(m), m, 0.0)
            e = np.exp(x - m)
            z = e.sum(axis=1, keepdims=True)
            with np.errstate(divide="ignore", invalid="ignore"):
                o = np.where(z > 0, (e @ v64[0, h]) / z, 0.0)
                l = np.where(z > 0, m + np.log(z), -np.inf)
            return o, l
        oA, lA = part(A)
        oB, lB = part(Bset)
        eA, eB = np.exp(lA), np.exp(lB)
        merged = (eA * oA + eB * oB) / (eA + eB)                # App. D merge
        np.testing.assert_allclose(out[0, h], merged, atol=1e-12, rtol=0)
        np.testing.assert_allclose(lse.reshape(B, Hq, n)[0, h], np.log(eA + eB)[:, 0], atol=1e-12)


# ---------------------------------------------------------------- P10 softcap
def test_p10_softcap_limits():
    B, Hq, Hkv, n, d, K = 1, 2, 1, 40, 8, 4
    q, k, v, c = rand_problem(41, B, Hq, Hkv, n, d, K)
    base = run_oracle(fo.Problem(B, Hq, Hkv, n, d, K, 2, 4), q, k, v, c)
    huge = run_oracle(fo.Problem(B, Hq, Hkv, n, d, K, 2, 4, softcap=1e6), q, k, v, c)
    np.testing.assert_allclose(huge[2], base[2], atol=1e-9)
    # a tiny cap flattens every allowed logit: uniform average over the allowed keys only
    tiny = run_oracle(fo.Problem(B, Hq, Hkv, n, d, K, 2, 4, softcap=1e-9), q, k, v, c,
                      want_probs=True)
    probs, pairs = tiny[5], tiny[4]
    for r in range(B * Hq * n):
        nz = probs[r] > 0
        assert nz.sum() == pairs[r]
        np.testing.assert_allclose(probs[r][nz], 1.0 / pairs[r], rtol=1e-6)
    # lse is bounded by cap + ln(pairs) because every logit lies in [-cap, cap]
    capped = run_oracle(fo.Problem(B, Hq, Hkv, n, d, K, 2, 4, softcap=0.5), q, k, v, c)
    assert np.all(capped[3] <= 0.5 + np.log(capped[4]) + 1e-12)
    assert np.all(capped[3] >= -0.5 + np.log(capped[4]) - 1e-12)


def test_p10_softcap_two_key_closed_form():
    # n=2, d=1: row 1 sees both keys; p0/p1 = exp(c tanh(s a k0 / c) - c tanh(s a k1 / c))
    a, k0, k1, s, cap = 1.5, 2.0, -0.75, 0.6, 1.25
    q = np.array([[[[0.3], [a]]]], dtype=np.float32)
    k = np.array([[[[k0], [k1]]]], dtype=np.float32)
    v = np.array([[[[1.0], [0.0]]]], dtype=np.float32)
    c = np.ones((1, 1, 1), dtype=np.float32)
    pb = fo.Problem(1, 1, 1, 2, 1, 1, 1, 1, scale=s, softcap=cap)
    mq, mk, out, lse, pairs = run_oracle(pb, q, k, v, c)
    ratio = math.exp(cap * math.tanh(s * a * k0 / cap) - cap * math.tanh(s * a * k1 / cap))
    assert abs(out[1, 0] - ratio / (1 + ratio)) < 1e-14
    assert out[0, 0] == 1.0


# ---------------------------------------------------------------- P11 retained fraction
def test_p11_expected_retained_fraction():
    n, d = 1536, 64
    for K, topk, expect in [(4, 2, 5 / 6), (8, 1, 1 / 8), (8, 2, 13 / 28)]:
        q, k, v, c = rand_problem(51 + K + topk, 1, 2, 2, n, d, K)
        pb = fo.Problem(1, 2, 2, n, d, K, topk, 1)       # window 1: only the diagonal is local
        mq = fo.membership(pb, q, c, True)
        mk = fo.membership(pb, k, c, False)
        allowed, _ = fo.pair_counts(pb, mq, mk)
        frac = (allowed.astype(np.float64) - n) / (n * (n - 1) / 2)
        assert np.all(np.abs(frac - expect) < 0.08), (K, topk, frac, expect)


# ---------------------------------------------------------------- P12 metamorphic
def test_p12_metamorphic():
    B, Hq, Hkv, n, d, K = 1, 4, 2, 48, 8, 4
    q, k, v, c = rand_problem(61, B, Hq, Hkv, n, d, K)
    pb = fo.Problem(B, Hq, Hkv, n, d, K, 2, 6)
    mq, mk, out, lse, pairs = run_oracle(pb, q, k, v, c)
    _, _, out2, lse2, _ = run_oracle(pb, q, k, (v * 4.0).astype(np.float32), c)
    np.testing.assert_allclose(out2, 4.0 * out, atol=1e-12)
    np.testing.assert_allclose(lse2, lse, atol=0)
    # GQA equals MHA with each KV head (and its centroids) repeated
    rep = [h // 2 for h in range(Hq)]
    pb_mha = fo.Problem(B, Hq, Hq, n, d, K, 2, 6)
    _, _, out3, lse3, pairs3 = run_oracle(pb_mha, q, k[:, rep].copy(), v[:, rep].copy(), c[rep].copy())
    np.testing.assert_allclose(out3, out, atol=0)
    assert np.array_equal(pairs3, pairs)
    # an explicit head map that permutes KV heads
    hm = np.array([1, 0, 1, 0], dtype=np.int32)
    pb_map = fo.Problem(B, Hq, Hkv, n, d, K, 2, 6, head_map=hm)
    _, _, out4, _, _ = run_oracle(pb_map, q, k, v, c)
    pb_m2 = fo.Problem(B, Hq, Hq, n, d, K, 2, 6)
    _, _, out5, _, _ = run_oracle(pb_m2, q, k[:, hm].copy(), v[:, hm].copy(), c[hm].copy())
    np.testing.assert_allclose(out4, out5, atol=0)


# ------------------------------------------------------- scores, top-k, lists
def test_scores_against_matmul_and_topk_against_argsort():
    B, Hq, Hkv, n, d, K = 2, 4, 2, 100, 64, 8
    for dtype in ("f32", "bf16"):
        q, k, v, c = rand_problem(71, B, Hq, Hkv, n, d, K, dtype=dtype)
        pb = fo.Problem(B, Hq, Hkv, n, d, K, 3, 4, dtype=dtype)
        sq = fo.scores(pb, q, c, True)
        sk = fo.scores(pb, k, c, False)
        c64 = c.astype(np.float64)
        want_q = np.einsum("bhnd,hkd->bhnk", brute.as_f64(q), c64[[h // 2 for h in range(Hq)]])
        want_k = np.einsum("bhnd,hkd->bhnk", brute.as_f64(k), c64)
        np.testing.assert_allclose(sq, want_q, atol=1e-12)
        np.testing.assert_allclose(sk, want_k, atol=1e-12)
        m = fo.topk_masks(pb, sq)
        order = np.argsort(-sq, axis=-1, kind="stable")[..., :3]
        want = np.zeros(m.shape, dtype=np.uint32)
        for t in range(3):
            want |= (np.uint32(1) << order[..., t].astype(np.uint32))
        assert np.array_equal(m, want)
        assert np.all(np.array([bin(x).count("1") for x in m.ravel()]) == 3)


def test_score_accumulation_order_is_sequential():
    # fp64 sum in index order: 1e16 + 1 + ... loses the ones only when added one by one
    d = 6
    x = np.array([[[[1.0, 1.0, 1.0, 1.0, 1.0, 1.0]]]], dtype=np.float32)
    c = np.array([[[1e16, 1, 1, 1, 1, -1e16], [1, 1, 1, 1, 1e16, -1e16]]], dtype=np.float32)
    pb = fo.Problem(1, 1, 1, 1, d, 2, 1, 1)
    s = fo.scores(pb, x, c, True)[0, 0, 0]
    big = float(np.float32(1e16))
    want0 = 0.0
    for t in [big, 1, 1, 1, 1, -big]:
        want0 = want0 + t
    want1 = 0.0
    for t in [1, 1, 1, 1, big, -big]:
        want1 = want1 + t
    assert s[0] == want0 and s[1] == want1 and want0 != want1


def test_topk_ties_lower_index_wins():
    sc = np.array([[[[1.0, 2.0, 2.0, 2.0], [0.0, 0.0, 0.0, 0.0], [3.0, 1.0, 3.0, 1.0]]]])
    pb = fo.Problem(1, 1, 1, 3, 4, 4, 2, 1)
    m = fo.topk_masks(pb, sc)
    assert list(m[0, 0]) == [0b0110, 0b0011, 0b0101]
    pb1 = fo.Problem(1, 1, 1, 3, 4, 4, 1, 1)
    assert list(fo.topk_masks(pb1, sc)[0, 0]) == [0b0010, 0b0001, 0b0001]


def test_scores_that_are_not_numbers_give_the_first_topk_groups():
    """The paper is silent on non-finite scores.  Reading: infinities are ordinary values of the ranking;
    a token with a NaN among its scores has no ranking and takes the first topk groups, so that every
    membership is a topk-subset (what the per-group lists of topk*n entries rest on)."""
    pb = fo.Problem(1, 1, 1, 6, 4, 4, 2, 4)
    inf, nan = float("inf"), float("nan")
    sc = np.array([[[[0.0, 3.0, nan, 1.0],            # a NaN: first two groups, not {1, 3} and not {1, 2, 3}
                     [nan, nan, nan, nan],
                     [inf, 1.0, inf, -inf],           # infinities rank; the tie between groups 0 and 2 is no issue
                     [-inf, -inf, -inf, 5.0],         # tie among -inf: lower index wins
                     [1.0, 2.0, 3.0, 4.0],
                     [inf, nan, 0.0, 0.0]]]])
    m = fo.topk_masks(pb, sc)[0, 0]
    assert [int(x) for x in m] == [0b0011, 0b0011, 0b0101, 0b1001, 0b1100, 0b0011]
    assert all(bin(int(x)).count("1") == 2 for x in m)
    # through the scoring itself: an Inf component against a zero centroid component makes a NaN score
    x = np.ones((1, 1, 6, 4), dtype=np.float32)
    x[0, 0, 2, 1] = inf
    c = np.array([[[1, 0, 0, 0], [0, 1, 0, 0], [0, 0, 1, 0], [0, 0, 0, 1]]], dtype=np.float32)
    assert int(fo.membership(pb, x, c, True)[0, 0, 2]) == 0b0011
    c2 = np.array([[[1, 1, 0, 0], [0, 1, 0, 0], [0, -1, 1, 0], [0, 1, 0, 1]]], dtype=np.float32)   # no zero against the Inf
    c2[c2 == 0] = 0.5
    assert int(fo.membership(pb, x, c2, True)[0, 0, 2]) == 0b0011   # +inf, +inf, -inf, +inf: groups 0 and 1


def test_group_lists_are_ascending_positions():
    rng = np.random.default_rng(5)
    B, H, n, K, topk = 2, 3, 200, 5, 2
    masks = np.zeros((B, H, n), dtype=np.uint32)
    for idx in itertools.product(range(B), range(H), range(n)):
        gs = rng.choice(K, size=topk, replace=False)
        masks[idx] = sum(1 << int(g) for g in gs)
    pb = fo.Problem(B, H, H, n, 4, K, topk, 1)
    counts, lists = fo.group_lists(pb, masks)
    assert np.all(counts.sum(axis=-1) == topk * n)
    for b in range(B):
        for h in range(H):
            off = 0
            for g in range(K):
                want = np.nonzero((masks[b, h] >> g) & 1)[0]
                assert counts[b, h, g] == len(want)
                assert np.array_equal(lists[b, h, off:off + len(want)], want)
                off += len(want)


def test_window_holds_exactly_w_keys():
    # all tokens in different groups from each other's keys: only the window survives
    n, K, w = 30, 2, 7
    q = np.zeros((1, 1, n, 2), dtype=np.float32); q[..., 0] = 1.0     # queries -> group 0
    k = np.zeros((1, 1, n, 2), dtype=np.float32); k[..., 1] = 1.0     # keys    -> group 1
    v = np.random.default_rng(0).standard_normal((1, 1, n, 2)).astype(np.float32)
    c = np.eye(2, dtype=np.float32)[None]
    pb = fo.Problem(1, 1, 1, n, 2, K, 1, w)
    mq, mk, out, lse, pairs = run_oracle(pb, q, k, v, c)
    assert np.array_equal(pairs, np.minimum(np.arange(n) + 1, w))
    # logits are all zero -> output is the plain mean of the last w values
    for i in range(n):
        lo = max(0, i - w + 1)
        np.testing.assert_allclose(out[i], v[0, 0, lo:i + 1].astype(np.float64).mean(axis=0), atol=1e-14)


def test_half_precision_storage_is_ieee_binary16():
    # Every one of the 65536 bit patterns, read by the oracle (score against the centroid [1.0] with
    # d = 1 is the stored value itself) and by numpy's float16: zeros, subnormals, normals, infinities, NaNs.
    bits = np.arange(65536, dtype=np.uint16).reshape(1, 1, 65536, 1)
    pb = fo.Problem(1, 1, 1, 65536, 1, 1, 1, 1, dtype="f16")
    got = fo.scores(pb, np.ascontiguousarray(bits), np.ones((1, 1, 1), dtype=np.float32), True).reshape(-1)
    want = bits.reshape(-1).view(np.float16).astype(np.float64)
    assert np.array_equal(np.isnan(got), np.isnan(want))
    ok = ~np.isnan(want)
    assert np.array_equal(got[ok], want[ok])                  # (-0 scores as +0: equal as numbers)


def test_half_precision_attention_matches_the_widened_inputs():
    # the same values handed over as fp16 bits and as fp32 give the same rows
    rng = np.random.default_rng(5)
    B, Hq, Hkv, n, d, K, topk, w = 1, 2, 1, 40, 8, 4, 2, 5
    q, k, v = (rng.standard_normal((B, H, n, d)).astype(np.float16) for H in (Hq, Hkv, Hkv))
    c = rng.standard_normal((Hkv, K, d)).astype(np.float32)
    outs = []
    for dtype, conv in (("f16", lambda a: np.ascontiguousarray(a.view(np.uint16))), ("f32", lambda a: a.astype(np.float32))):
        pb = fo.Problem(B, Hq, Hkv, n, d, K, topk, w, dtype=dtype)
        mq = fo.membership(pb, conv(q), c, True)
        mk = fo.membership(pb, conv(k), c, False)
        outs.append(fo.attn_rows(pb, conv(q), conv(k), conv(v), mq, mk))
    for a, b in zip(outs[0], outs[1]):
        assert np.array_equal(a, b)
