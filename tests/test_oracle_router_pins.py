"""Pins of the router oracle (Sec. 2 Eq. 1 + Sinkhorn recipe) against things other than itself.

R1 the projection against a library matmul (and exactly, on small integers);
R2 the sequential accumulation order of the inner product; R3 no normalisation = plain top-k of (h W_g) C^T / tau;
R4 a literal Python transcription of the recipe without the max shift on a tiny case;
R5 Sinkhorn invariants: rows sum to one, cross-ratios of exp(S/tau) are preserved
(diagonal scaling), columns balance to n/K in the limit; R6 degenerate cases
(equal centroids, K = 1, topk = K); R7 batch elements are independent; R8 the
balancing claim of the iteration-count ablation (App., Sinkhorn iterations) in its
weak form: more iterations never leave a dominant group more dominant than plain top-1.
"""
import math

import numpy as np
import pytest
import torch

from oracle import focus_oracle as fo


def rand_router(seed, B, n, dm, dg, K, spread=1.0):
    rng = np.random.default_rng(seed)
    h = rng.standard_normal((B, n, dm)).astype(np.float32)
    wg = (rng.standard_normal((dm, dg)) / math.sqrt(dm)).astype(np.float32)
    c = (spread * rng.standard_normal((K, dg))).astype(np.float32)
    return h, wg, c


def mask_of(idx):
    m = 0
    for g in idx:
        m |= 1 << int(g)
    return m


# ---------------------------------------------------------------- R1 / R2 projection
def test_r1_projection_matches_matmul():
    h, wg, c = rand_router(1, 2, 77, 200, 16, 8)
    _, z, _ = fo.route(h, wg, c, 2, iters=0, want_soft=True)
    ref = torch.from_numpy(h).double() @ torch.from_numpy(wg).double()
    assert np.abs(z - ref.numpy()).max() < 1e-13


def test_r1_projection_exact_on_small_integers():
    rng = np.random.default_rng(2)
    h = rng.integers(-8, 9, size=(1, 33, 130)).astype(np.float32)
    wg = rng.integers(-8, 9, size=(130, 5)).astype(np.float32)
    c = rng.integers(-4, 5, size=(6, 5)).astype(np.float32)
    _, z, g = fo.route(h, wg, c, 2, tau=0.5, iters=0, want_soft=True)
    zi = h.astype(np.int64) @ wg.astype(np.int64)
    assert np.array_equal(z, zi.astype(np.float64))
    assert np.array_equal(g, (zi @ c.astype(np.int64).T).astype(np.float64) / 0.5)


def test_r1_bf16_hidden_is_widened_exactly():
    h, wg, c = rand_router(3, 1, 40, 96, 16, 8)
    hb = torch.from_numpy(h).to(torch.bfloat16)
    bits = hb.view(torch.int16).numpy().view(np.uint16)
    _, z, _ = fo.route(bits, wg, c, 2, iters=0, dtype="bf16", want_soft=True)
    ref = hb.double() @ torch.from_numpy(wg).double()
    assert np.abs(z - ref.numpy()).max() < 1e-13


def test_r2_accumulation_is_sequential_in_index_order():
    """Eq. 1 is a plain inner product; the oracle adds its terms one by one, t = 0 .. d_model-1.

    Checked against math.fsum-free, exactly representable cases that tell the sequential order
    from a blocked or pairwise one: 2^53 followed by ones loses every one when they are added
    singly (round to even), and keeps them when they are first summed among themselves."""
    dm = 192
    wg = np.ones((dm, 1), dtype=np.float32)
    c = np.ones((1, 1), dtype=np.float32)
    h = np.zeros((1, 1, dm), dtype=np.float32)
    h[0, 0, 0] = 2.0 ** 53
    h[0, 0, 64:192] = 1.0                       # two whole blocks of 64 ones: any 64-blocked sum keeps them
    _, z, _ = fo.route(h, wg, c, 1, iters=0, want_soft=True)
    assert z[0, 0, 0] == 2.0 ** 53
    # the ones first, the large term last: every term survives
    h2 = np.zeros((1, 1, dm), dtype=np.float32)
    h2[0, 0, :191] = 1.0
    h2[0, 0, 191] = 2.0 ** 53
    _, z2, _ = fo.route(h2, wg, c, 1, iters=0, want_soft=True)
    assert z2[0, 0, 0] == 2.0 ** 53 + 192.0              # 191 + 2^53 is a tie: rounds to the even neighbour
    # a python left-to-right float sum is the same recipe (floats are fp64, products here are exact)
    rng = np.random.default_rng(12)
    h3 = rng.standard_normal((1, 3, 150)).astype(np.float32)
    w3 = rng.standard_normal((150, 2)).astype(np.float32)
    _, z3, _ = fo.route(h3, w3, np.ones((1, 2), dtype=np.float32), 1, iters=0, want_soft=True)
    for i in range(3):
        for j in range(2):
            acc = 0.0
            for t in range(150):
                acc += float(h3[0, i, t]) * float(w3[t, j])
            assert z3[0, i, j] == acc


def test_router_width_beyond_the_oracle_buffer_is_refused():
    h, wg, c = rand_router(13, 1, 4, 16, 257, 2)
    with pytest.raises(Exception):
        fo.route(h, wg, c, 1, iters=0)


# ---------------------------------------------------------------- R3 plain top-k
@pytest.mark.parametrize("topk", [1, 2, 3])
def test_r3_no_sinkhorn_is_plain_topk(topk):
    h, wg, c = rand_router(4, 2, 301, 64, 16, 8)
    masks, z, g = fo.route(h, wg, c, topk, tau=0.25, iters=0, want_soft=True)
    s = (h.astype(np.float64) @ wg.astype(np.float64)) @ c.astype(np.float64).T
    assert np.abs(g - s / 0.25).max() < 1e-12
    order = np.argsort(-g, axis=-1, kind="stable")[..., :topk]
    want = np.array([[mask_of(order[b, i]) for i in range(g.shape[1])] for b in range(g.shape[0])], dtype=np.uint32)
    assert np.array_equal(masks, want)


# ---------------------------------------------------------------- R4 literal recipe
def literal_sinkhorn(S, tau, iters):
    n, K = len(S), len(S[0])
    Q = [[math.exp(S[i][g] / tau) for g in range(K)] for i in range(n)]
    for _ in range(iters):
        col = [sum(Q[i][g] for i in range(n)) for g in range(K)]
        Q = [[Q[i][g] / col[g] for g in range(K)] for i in range(n)]
        row = [sum(Q[i][g] for g in range(K)) for i in range(n)]
        Q = [[Q[i][g] / row[i] for g in range(K)] for i in range(n)]
    return np.array(Q)


@pytest.mark.parametrize("iters", [1, 3, 10])
def test_r4_literal_recipe_on_tiny_case(iters):
    h, wg, c = rand_router(5, 1, 7, 12, 4, 3)
    masks, z, g = fo.route(h, wg, c, 1, tau=0.1, iters=iters, want_soft=True)
    S = (z[0] @ c.astype(np.float64).T).tolist()
    want = literal_sinkhorn(S, 0.1, iters)
    assert np.abs(g[0] - want).max() < 1e-12
    assert np.array_equal(masks[0], np.array([1 << int(a) for a in want.argmax(-1)], dtype=np.uint32))


# ---------------------------------------------------------------- R5 invariants
def test_r5_rows_sum_to_one_and_cross_ratios():
    h, wg, c = rand_router(6, 1, 120, 48, 16, 8, spread=0.3)
    tau = 0.1
    _, z, g = fo.route(h, wg, c, 2, tau=tau, iters=10, want_soft=True)
    assert np.abs(g.sum(-1) - 1.0).max() < 1e-12
    assert (g > 0).all()
    S = z[0] @ c.astype(np.float64).T
    L = np.log(g[0])
    rng = np.random.default_rng(0)
    for _ in range(200):
        i, j = rng.integers(0, 120, 2)
        a, b = rng.integers(0, 8, 2)
        lhs = L[i, a] + L[j, b] - L[i, b] - L[j, a]
        rhs = (S[i, a] + S[j, b] - S[i, b] - S[j, a]) / tau
        assert abs(lhs - rhs) < 1e-8 * max(1.0, abs(rhs))


def test_r5_columns_balance_in_the_limit():
    h, wg, c = rand_router(7, 2, 400, 32, 8, 4, spread=0.2)
    _, _, g = fo.route(h, wg, c, 1, tau=0.5, iters=300, want_soft=True)
    assert np.abs(g.sum(1) - 400 / 4).max() < 1e-6
    # one iteration ends on the row step: rows are exact, columns are not yet
    _, _, g1 = fo.route(h, wg, c, 1, tau=0.5, iters=1, want_soft=True)
    assert np.abs(g1.sum(-1) - 1.0).max() < 1e-12
    assert np.abs(g1.sum(1) - 100.0).max() > 1e-3


# ---------------------------------------------------------------- R6 degenerate cases
@pytest.mark.parametrize("iters", [0, 5])
def test_r6_equal_centroids_tie_to_lowest_indices(iters):
    h, wg, _ = rand_router(8, 1, 50, 16, 4, 6)
    c = np.tile(np.array([[0.5, -1.0, 2.0, 0.25]], dtype=np.float32), (6, 1))
    masks, _, g = fo.route(h, wg, c, 3, iters=iters, want_soft=True)
    assert (masks == 0b111).all()
    if iters:
        assert np.abs(g - 1.0 / 6).max() < 1e-15


def test_r6_single_group_and_full_topk():
    h, wg, c = rand_router(9, 1, 20, 16, 4, 1)
    assert (fo.route(h, wg, c, 1, iters=10) == 1).all()
    h, wg, c = rand_router(9, 1, 20, 16, 4, 5)
    assert (fo.route(h, wg, c, 5, iters=10) == 31).all()


def test_r6_common_offset_cancels_and_cannot_overflow():
    # A score offset shared by the whole sequence (here +100, i.e. +1000 after the division by tau, far past
    # the overflow point of exp) is divided out by the first column step: same soft assignment as without it.
    h, wg, c = rand_router(10, 1, 64, 16, 4, 4, spread=0.3)
    _, _, g0 = fo.route(h, wg, c, 1, tau=0.1, iters=10, want_soft=True)
    h2 = np.concatenate([h, np.ones((1, 64, 1), np.float32)], axis=-1)
    wg2 = np.concatenate([np.concatenate([wg, np.zeros((16, 1), np.float32)], axis=1),
                          np.array([[0, 0, 0, 0, 100.0]], np.float32)], axis=0)
    c2 = np.concatenate([c, np.ones((4, 1), np.float32)], axis=1)
    _, _, g1 = fo.route(h2, wg2, c2, 1, tau=0.1, iters=10, want_soft=True)
    assert np.isfinite(g1).all()
    assert np.abs(g1 - g0).max() < 1e-9


# ---------------------------------------------------------------- R7 batch independence
def test_r7_batch_elements_are_independent():
    h, wg, c = rand_router(11, 3, 90, 40, 16, 8)
    both = fo.route(h, wg, c, 2, iters=10)
    for b in range(3):
        assert np.array_equal(both[b:b + 1], fo.route(h[b:b + 1], wg, c, 2, iters=10))


# ---------------------------------------------------------------- R8 balancing
def test_r8_sinkhorn_reduces_dominance():
    rng = np.random.default_rng(12)
    K = dg = 8
    wg = np.eye(dg, dtype=np.float32)
    c = rng.standard_normal((K, dg)).astype(np.float32)
    h = (0.5 * rng.standard_normal((1, 2000, dg)) + 0.8 * c[0]).astype(np.float32)   # every token leans to group 0

    def top_share(iters):
        m = fo.route(h, wg, c, 1, tau=0.1, iters=iters)
        return np.bincount(np.log2(m.ravel()).astype(int), minlength=K).max() / m.size

    plain, s10, s50 = top_share(0), top_share(10), top_share(50)
    assert plain > 0.5
    assert s50 <= s10 <= plain
    assert s50 < 0.2                                              # 1/K = 0.125 is perfect balance


# ---------------------------------------------------------------- token masks feed the attention oracle
def test_broadcast_masks_to_heads():
    pb = fo.Problem(2, 4, 2, 33, 8, 4, 2, 4)
    tm = np.random.default_rng(0).integers(1, 16, size=(2, 33)).astype(np.uint32)
    mq, mk = fo.broadcast_masks(pb, tm)
    assert mq.shape == (2, 4, 33) and mk.shape == (2, 2, 33)
    assert (mq == tm[:, None, :]).all() and (mk == tm[:, None, :]).all()
