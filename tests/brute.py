"""A second, deliberately naive statement of Focus attention used only to pin the
oracle on tiny problems (pure Python loops, memberships as sorted id lists,
probabilities through numpy.longdouble).  Written independently of oracle/.

Follows App. D Eq. 3 generalised to top-k sets (Sec. 2, "Efficiency at
inference"): a pair is attended when it is causal and either within the window
or the two tokens have a group in common.
"""
import math

import numpy as np


def bf16_bits_to_float(u16):
    u32 = np.asarray(u16, dtype=np.uint32) << np.uint32(16)
    return u32.view(np.float32).astype(np.float64)


def as_f64(x):
    x = np.asarray(x)
    if x.dtype == np.uint16:
        return bf16_bits_to_float(x)
    return x.astype(np.float64)


def member_ids(vec, cents, topk):
    """ids of the topk best-scoring centroids, lower id first on ties, sorted ascending."""
    K = cents.shape[0]
    s = []
    for g in range(K):
        acc = 0.0
        for t in range(len(vec)):
            acc += float(vec[t]) * float(cents[g][t])
        s.append(acc)
    order = sorted(range(K), key=lambda g: (-s[g], g))
    return sorted(order[:topk])


def attention(q, k, v, cents, topk, window, causal=True, head_map=None, scale=None, softcap=0.0):
    """q [B,Hq,n,d], k/v [B,Hkv,n,d], cents [Hkv,K,d] (float arrays).
    Returns out [B,Hq,n,d], lse [B,Hq,n], pairs [B,Hq,n], ids_q, ids_k (nested lists)."""
    q, k, v = as_f64(q), as_f64(k), as_f64(v)
    cents = np.asarray(cents, dtype=np.float64)
    B, Hq, n, d = q.shape
    Hkv = k.shape[1]
    if scale is None:
        scale = 1.0 / math.sqrt(d)
    out = np.zeros((B, Hq, n, d))
    lse = np.zeros((B, Hq, n))
    pairs = np.zeros((B, Hq, n), dtype=np.int64)
    ids_q = [[[None] * n for _ in range(Hq)] for _ in range(B)]
    ids_k = [[[None] * n for _ in range(Hkv)] for _ in range(B)]
    for b in range(B):
        for hk in range(Hkv):
            for j in range(n):
                ids_k[b][hk][j] = member_ids(k[b, hk, j], cents[hk], topk)
        for h in range(Hq):
            hk = head_map[h] if head_map is not None else h // (Hq // Hkv)
            for i in range(n):
                gi = member_ids(q[b, h, i], cents[hk], topk)
                ids_q[b][h][i] = gi
                logits = []
                keys = []
                for j in range(n):
                    if causal and j > i:
                        continue
                    near = (i - j < window) if causal else (abs(i - j) < window)
                    common = len(set(gi).intersection(ids_k[b][hk][j])) > 0
                    if not (near or common):
                        continue
                    x = scale * sum(float(q[b, h, i, t]) * float(k[b, hk, j, t]) for t in range(d))
                    if softcap > 0:
                        x = softcap * math.tanh(x / softcap)
                    logits.append(x)
                    keys.append(j)
                lg = np.array(logits, dtype=np.longdouble)
                mx = lg.max()
                e = np.exp(lg - mx)
                z = e.sum()
                p = e / z
                acc = np.zeros(d, dtype=np.longdouble)
                for pj, j in zip(p, keys):
                    acc += pj * v[b, hk, j].astype(np.longdouble)
                out[b, h, i] = acc.astype(np.float64)
                lse[b, h, i] = float(mx + np.log(z))
                pairs[b, h, i] = len(keys)
    return out, lse, pairs, ids_q, ids_k


def ids_to_mask(ids):
    m = 0
    for g in ids:
        m |= 1 << g
    return m
