"""Pins of the oracle's two-set decomposition (App. D: A = pairs that share a group, B = window pairs
that share none, log-sum-exp merge) against things other than itself.

S1 each set against an independent numpy masked softmax; S2 the sets are disjoint and cover the mask
(probability supports and pair counts); S3 merge(A, B) equals the attention over the whole mask — the
exactness App. D states; S4 degenerate cases: K = 1 (A is dense causal attention, checked against
torch SDPA; B is empty), window 1 with one assignment per token (B empty, A = everything), a row whose
set is empty; S5 the merge formula against closed forms.
"""
import math

import numpy as np
import pytest
import torch

from oracle import focus_oracle as fo
from tests.test_oracle_pins import rand_problem, run_oracle


def numpy_part(q, k, v, mask, scale):
    x = np.where(mask, (q @ k.T) * scale, -np.inf)
    m = x.max(axis=1, keepdims=True)
    m = np.where(np.isfinite(m), m, 0.0)
    e = np.exp(x - m)
    z = e.sum(axis=1, keepdims=True)
    with np.errstate(divide="ignore", invalid="ignore"):
        o = np.where(z > 0, (e @ v) / z, 0.0)
        l = np.where(z > 0, m + np.log(z), -np.inf)[:, 0]
    return o, l, mask.sum(axis=1)


@pytest.mark.parametrize("topk,w,same_vectors", [(1, 5, True), (1, 5, False), (2, 3, False), (2, 64, False), (3, 1, False)])
def test_s1_s2_s3_sets_and_merge(topk, w, same_vectors):
    B, Hq, Hkv, n, d, K = 1, 4, 2, 48, 8, 6
    q, k, v, c = rand_problem(71, B, Hq, Hkv, n, d, K)
    if same_vectors:
        Hq = Hkv
        q = k.copy()
    pb = fo.Problem(B, Hq, Hkv, n, d, K, topk, w)
    mq, mk, out, lse, pairs = run_oracle(pb, q, k, v, c)
    oA, lA, pA, prA = fo.attn_rows(pb, q, k, v, mq, mk, want_probs=True, pair_set="A")
    oB, lB, pB, prB = fo.attn_rows(pb, q, k, v, mq, mk, want_probs=True, pair_set="B")
    _, _, _, pr = fo.attn_rows(pb, q, k, v, mq, mk, want_probs=True)
    # S2: disjoint supports that cover the support of the whole mask; counts add up
    assert not np.any((prA > 0) & (prB > 0))
    assert np.array_equal((prA > 0) | (prB > 0), pr > 0)
    assert np.array_equal(pA + pB, pairs)
    # S1: each set against numpy
    ii, jj = np.meshgrid(np.arange(n), np.arange(n), indexing="ij")
    G = Hq // Hkv
    for h in range(Hq):
        share = (mq[0, h][:, None] & mk[0, h // G][None, :]) != 0
        A = (jj <= ii) & share
        Bm = (jj <= ii) & (ii - jj < w) & ~share
        q64, k64, v64 = q[0, h].astype(np.float64), k[0, h // G].astype(np.float64), v[0, h // G].astype(np.float64)
        for mask, o_got, l_got, p_got in ((A, oA, lA, pA), (Bm, oB, lB, pB)):
            o_ref, l_ref, cnt = numpy_part(q64, k64, v64, mask, 1.0 / math.sqrt(d))
            sl = slice(h * n, (h + 1) * n)
            np.testing.assert_allclose(o_got[sl], o_ref, atol=1e-12, rtol=0)
            assert np.array_equal(np.isfinite(l_got[sl]), np.isfinite(l_ref))
            fin = np.isfinite(l_ref)
            np.testing.assert_allclose(l_got[sl][fin], l_ref[fin], atol=1e-12)
            assert np.array_equal(p_got[sl], cnt)
    # S3: the merge is exact
    om, lm = fo.merge(oA, lA, oB, lB)
    np.testing.assert_allclose(om, out, atol=1e-12, rtol=0)
    np.testing.assert_allclose(lm, lse, atol=1e-12, rtol=0)
    cos = (om * out).sum() / (np.linalg.norm(om) * np.linalg.norm(out))
    assert cos > 1 - 1e-12                     # the paper quotes cosine similarity 1.0000 for this check


def test_s4_single_group_is_dense_causal():
    B, H, n, d = 1, 2, 33, 16
    q, k, v, c = rand_problem(72, B, H, H, n, d, 1)
    pb = fo.Problem(B, H, H, n, d, 1, 1, 4)
    mq, mk, out, lse, pairs = run_oracle(pb, q, k, v, c)
    oA, lA, pA = fo.attn_rows(pb, q, k, v, mq, mk, pair_set="A")
    oB, lB, pB = fo.attn_rows(pb, q, k, v, mq, mk, pair_set="B")
    ref = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(q).double(), torch.from_numpy(k).double(), torch.from_numpy(v).double(), is_causal=True)
    np.testing.assert_allclose(oA.reshape(B, H, n, d), ref.numpy(), atol=1e-12)
    assert (pB == 0).all() and (oB == 0).all() and np.isneginf(lB).all()
    assert np.array_equal(pA, pairs)


def test_s4_empty_rows():
    # per-head membership: a query whose own key sits in another group has no pair in A at position 0
    B, H, n, d, K = 1, 1, 20, 8, 4
    q, k, v, c = rand_problem(73, B, H, H, n, d, K)
    pb = fo.Problem(B, H, H, n, d, K, 1, 3)
    mq, mk, *_ = run_oracle(pb, q, k, v, c)
    mq = mq.copy(); mk = mk.copy()
    mq[0, 0, 0] = 1; mk[0, 0, 0] = 2                    # token 0: query in group 0, key in group 1
    oA, lA, pA = fo.attn_rows(pb, q, k, v, mq, mk, pair_set="A")
    oB, lB, pB = fo.attn_rows(pb, q, k, v, mq, mk, pair_set="B")
    assert pA[0] == 0 and (oA[0] == 0).all() and lA[0] == -np.inf
    assert pB[0] == 1 and np.allclose(oB[0], v[0, 0, 0])   # its only pair is itself, in B
    o, l, p = fo.attn_rows(pb, q, k, v, mq, mk)
    om, lm = fo.merge(oA, lA, oB, lB)
    np.testing.assert_allclose(om, o, atol=1e-12)
    np.testing.assert_allclose(lm, l, atol=1e-12)


def test_s5_merge_closed_forms():
    oa = np.array([[1.0, 2.0], [0.0, 0.0], [3.0, 3.0], [5.0, 5.0]])
    ob = np.array([[3.0, 6.0], [4.0, 4.0], [0.0, 0.0], [7.0, 7.0]])
    la = np.array([0.0, -np.inf, 2.0, 1000.0])
    lb = np.array([0.0, 1.0, -np.inf, 1000.0 + math.log(3.0)])
    o, l = fo.merge(oa, la, ob, lb)
    np.testing.assert_allclose(o[0], [2.0, 4.0])                 # equal weights: the mean
    np.testing.assert_allclose(l[0], math.log(2.0))
    np.testing.assert_allclose(o[1], [4.0, 4.0]); assert l[1] == 1.0     # an empty set weighs nothing
    np.testing.assert_allclose(o[2], [3.0, 3.0]); assert l[2] == 2.0
    np.testing.assert_allclose(o[3], [6.5, 6.5])                 # weights 1:3, no overflow at lse = 1000
    np.testing.assert_allclose(l[3], 1000.0 + math.log(4.0))
    o, l = fo.merge(oa[:1], np.array([-np.inf]), ob[:1], np.array([-np.inf]))
    assert (o == 0).all() and l[0] == -np.inf
