"""Pins of the oracle's soft-gated attention (Sec. 2 Eq. 2) against things other than itself:
a textbook dense causal attention written with numpy matrices, a brute-force evaluation of the
equation on tiny inputs, closed forms of two- and three-token rows, and the limits of the gate."""
import numpy as np
import pytest

from oracle import focus_oracle as fo


def draw(rng, B, Hq, Hkv, n, d, K):
    q = rng.standard_normal((B, Hq, n, d)).astype(np.float32)
    k = rng.standard_normal((B, Hkv, n, d)).astype(np.float32)
    v = rng.standard_normal((B, Hkv, n, d)).astype(np.float32)
    g = rng.random((B, n, K)).astype(np.float32)
    g /= g.sum(axis=-1, keepdims=True)
    return q, k, v, g.astype(np.float32)


def dense_causal(q, k, v, logits_of):
    """softmax over j <= i of logits_of(b, h) [n,n] (numpy, matrix form), times v."""
    B, Hq, n, d = q.shape
    G = Hq // k.shape[1]
    out = np.zeros((B, Hq, n, d))
    lse = np.zeros((B, Hq, n))
    for b in range(B):
        for h in range(Hq):
            x = logits_of(b, h).astype(np.float64)
            x = np.where(np.tril(np.ones((n, n), dtype=bool)), x, -np.inf)
            m = x.max(axis=1, keepdims=True)
            e = np.exp(x - m)
            s = e.sum(axis=1, keepdims=True)
            out[b, h] = (e / s) @ v[b, h // G].astype(np.float64)
            lse[b, h] = (m + np.log(s))[:, 0]
    return out.reshape(-1, d), lse.reshape(-1)


def test_g1_window_covering_the_sequence_is_plain_causal_attention():
    rng = np.random.default_rng(11)
    B, Hq, Hkv, n, d, K = 2, 4, 2, 33, 16, 4
    q, k, v, g = draw(rng, B, Hq, Hkv, n, d, K)
    pb = fo.Problem(B, Hq, Hkv, n, d, K, 2, n)               # every pair local: all gates are 1
    out, lse = fo.soft_rows(pb, 7.0, g, q, k, v)
    want, wlse = dense_causal(q, k, v, lambda b, h: (q[b, h].astype(np.float64) @ k[b, h // 2].astype(np.float64).T) / np.sqrt(d))
    assert np.abs(out - want).max() < 1e-12 and np.abs(lse - wlse).max() < 1e-12


@pytest.mark.parametrize("lam,w", [(0.0, 3), (5.0, 1), (-2.0, 4), (40.0, 2)])
def test_g2_matrix_form_of_the_equation(lam, w):
    rng = np.random.default_rng(12)
    B, Hq, Hkv, n, d, K = 1, 2, 1, 21, 8, 3
    q, k, v, g = draw(rng, B, Hq, Hkv, n, d, K)
    pb = fo.Problem(B, Hq, Hkv, n, d, K, 1, w)

    def logits(b, h):
        s = (q[b, h].astype(np.float64) @ k[b, 0].astype(np.float64).T) / np.sqrt(d)
        aff = g[b].astype(np.float64) @ g[b].astype(np.float64).T
        i, j = np.indices((n, n))
        local = (j <= i) & (j > i - w)
        gate = np.where(local, 1.0, 1.0 / (1.0 + np.exp(-lam * aff)))
        return s * gate

    out, lse = fo.soft_rows(pb, lam, g, q, k, v)
    want, wlse = dense_causal(q, k, v, logits)
    assert np.abs(out - want).max() < 1e-12 and np.abs(lse - wlse).max() < 1e-12


def test_g3_two_token_closed_form():
    # n = 2, w = 1: row 1 sees key 0 through the gate and itself at full strength
    d, K = 2, 2
    q = np.zeros((1, 1, 2, d), np.float32); k = np.zeros_like(q); v = np.zeros_like(q)
    q[0, 0, 1] = [2.0, 0.0]
    k[0, 0, 0] = [3.0, 0.0]; k[0, 0, 1] = [1.0, 0.0]
    v[0, 0, 0] = [1.0, 0.0]; v[0, 0, 1] = [0.0, 1.0]
    g = np.array([[[0.5, 0.5], [1.0, 0.0]]], np.float32)       # g_1 . g_0 = 0.5
    lam = 2.0
    pb = fo.Problem(1, 1, 1, 2, d, K, 1, 1, scale=1.0)
    out, lse, probs = fo.soft_rows(pb, lam, g, q, k, v, want_probs=True)
    gate = 1.0 / (1.0 + np.exp(-lam * 0.5))
    x0, x1 = 6.0 * gate, 2.0
    p0 = np.exp(x0) / (np.exp(x0) + np.exp(x1))
    assert abs(probs[1, 0] - p0) < 1e-14 and abs(probs[1, 1] - (1 - p0)) < 1e-14
    assert np.allclose(out[1], [p0, 1 - p0], atol=1e-14)
    assert abs(lse[1] - np.log(np.exp(x0) + np.exp(x1))) < 1e-13
    assert np.allclose(out[0], [1.0, 0.0]) and abs(lse[0] - 0.0) < 1e-15     # row 0: itself only, q_0 = 0


def test_g4_gate_limits():
    rng = np.random.default_rng(13)
    B, Hq, Hkv, n, d, K, w = 1, 2, 2, 30, 8, 4, 3
    q, k, v, _ = draw(rng, B, Hq, Hkv, n, d, K)
    grp = rng.integers(0, K, size=(B, n))
    g = np.eye(K, dtype=np.float32)[grp]                        # one-hot: affinity 1 (same group) or 0
    pb = fo.Problem(B, Hq, Hkv, n, d, K, 1, w)
    # a steep gate: same-group distant pairs at full strength, the others at exactly half (sigmoid(0))
    out, lse = fo.soft_rows(pb, 800.0, g, q, k, v)

    def logits(b, h):
        s = (q[b, h].astype(np.float64) @ k[b, h].astype(np.float64).T) / np.sqrt(d)
        i, j = np.indices((n, n))
        local = (j <= i) & (j > i - w)
        same = grp[b][:, None] == grp[b][None, :]
        return s * np.where(local | same, 1.0, 0.5)

    want, wlse = dense_causal(q, k, v, logits)
    assert np.abs(out - want).max() < 1e-12 and np.abs(lse - wlse).max() < 1e-12
    # a very negative slope closes same-group gates (logit 0, weight e^0: the pair is not removed)
    out2, _ = fo.soft_rows(pb, -800.0, g, q, k, v)

    def logits2(b, h):
        s = (q[b, h].astype(np.float64) @ k[b, h].astype(np.float64).T) / np.sqrt(d)
        i, j = np.indices((n, n))
        local = (j <= i) & (j > i - w)
        same = grp[b][:, None] == grp[b][None, :]
        return s * np.where(local, 1.0, np.where(same, 0.0, 0.5))

    want2, _ = dense_causal(q, k, v, logits2)
    assert np.abs(out2 - want2).max() < 1e-12


def test_g5_rows_are_convex_combinations_and_sampled_rows_match():
    rng = np.random.default_rng(14)
    B, Hq, Hkv, n, d, K, w = 2, 4, 2, 40, 8, 5, 6
    q, k, v, g = draw(rng, B, Hq, Hkv, n, d, K)
    pb = fo.Problem(B, Hq, Hkv, n, d, K, 2, w)
    out, lse, probs = fo.soft_rows(pb, 3.0, g, q, k, v, want_probs=True)
    assert np.abs(probs.sum(axis=1) - 1.0).max() < 1e-13
    i = np.tile(np.arange(n), B * Hq)
    assert all(probs[r, i[r] + 1:].sum() == 0.0 for r in range(probs.shape[0]))   # causal
    rows = np.array([[1, 3, 17], [0, 0, 0], [1, 2, 39]], dtype=np.int32)
    o2, l2 = fo.soft_rows(pb, 3.0, g, q, k, v, rows=rows)
    for t, (b, h, ii) in enumerate(rows):
        r = (b * Hq + h) * n + ii
        assert np.array_equal(o2[t], out[r]) and l2[t] == lse[r]


def test_g6_bf16_and_gqa_head_map():
    rng = np.random.default_rng(15)
    B, Hq, Hkv, n, d, K, w = 1, 3, 2, 25, 8, 4, 4
    q, k, v, g = draw(rng, B, Hq, Hkv, n, d, K)
    bits = lambda a: (a.view(np.uint32) >> 16).astype(np.uint16)            # truncation to bf16 storage
    back = lambda u: (u.astype(np.uint32) << 16).view(np.float32)
    hm = [1, 0, 1]
    pb16 = fo.Problem(B, Hq, Hkv, n, d, K, 2, w, dtype="bf16", head_map=hm)
    out, lse = fo.soft_rows(pb16, 4.0, g, bits(q), bits(k), bits(v))
    qf, kf, vf = back(bits(q)), back(bits(k)), back(bits(v))

    def logits(b, h):
        s = (qf[b, h].astype(np.float64) @ kf[b, hm[h]].astype(np.float64).T) / np.sqrt(d)
        aff = g[b].astype(np.float64) @ g[b].astype(np.float64).T
        i, j = np.indices((n, n))
        local = (j <= i) & (j > i - w)
        return s * np.where(local, 1.0, 1.0 / (1.0 + np.exp(-4.0 * aff)))

    want = np.zeros((B, Hq, n, d))
    for h in range(Hq):
        x = np.where(np.tril(np.ones((n, n), dtype=bool)), logits(0, h), -np.inf)
        e = np.exp(x - x.max(axis=1, keepdims=True))
        want[0, h] = (e / e.sum(axis=1, keepdims=True)) @ vf[0, hm[h]].astype(np.float64)
    assert np.abs(out - want.reshape(-1, d)).max() < 1e-12
